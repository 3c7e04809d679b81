"""Proxy-query partitions (paper Section 4.2): the executor holding the OLD part of the cache
works one layer ahead and therefore uses an approximate query; the recent part uses the true
query.  The ABI expresses this as two hg_attn_partial calls with two descriptors whose triples
are merged together.  The result is an approximation of full attention, but GPU and oracle must
still agree on it exactly (same inputs, same arithmetic), and with an exact proxy it must fall
back to the unsplit result."""
import numpy as np
import pytest
import torch

import oracle
import paper_2604_18529_amd as hg
from paper_2604_18529_amd import workloads as W

from parity_utils import check_out, check_triples, kv_np, to_np

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _hybrid(w, q_old, old_ranges, new_ranges, gp):
    """GPU: partial(old ranges, proxy q) + partial(new ranges, true q) -> merge."""
    m1, l1, o1 = hg.hg_attn_partial(q_old, w.k, w.v, w.seq_lens, old_ranges, w.scale)
    m2, l2, o2 = hg.hg_attn_partial(w.q, w.k, w.v, w.seq_lens, new_ranges, w.scale)
    # triples ordered per sequence: old, new
    B = len(old_ranges)
    idx = torch.arange(2 * B, device=DEV).reshape(2, B).t().reshape(-1)
    m = torch.cat([m1, m2])[idx].contiguous()
    l = torch.cat([l1, l2])[idx].contiguous()
    o = torch.cat([o1, o2])[idx].contiguous()
    return (m, l, o), hg.hg_attn_merge(m, l, o, gp)


def _hybrid_oracle(w, q_old, old_ranges, new_ranges, gp):
    kn, vn = kv_np(w)
    a = oracle.attn_partial(to_np(q_old), kn, vn, w.seq_lens, w.scale, old_ranges)
    b = oracle.attn_partial(to_np(w.q), kn, vn, w.seq_lens, w.scale, new_ranges)
    B = len(old_ranges)
    idx = np.arange(2 * B).reshape(2, B).T.reshape(-1)
    m, l, o = (np.concatenate([x, y])[idx] for x, y in zip(a, b))
    return (m, l, o), oracle.attn_merge(m, l, o, gp)


@pytest.mark.parametrize("group", [1, 8])
@pytest.mark.parametrize("cosine", [1.0, 0.98, 0.9])
def test_proxy_query_partitions(group, cosine):
    spec = W.WorkloadSpec("proxy", 3, 2 * group, 2, 128, "f16", 1500, 4000, "none", seed=41 + group)
    w = W.make_workload(spec, DEV)
    old = [(b, 0, int(0.7 * n)) for b, n in enumerate(w.seq_lens)]   # evicted first: oldest tokens
    new = [(b, int(0.7 * n), int(n)) for b, n in enumerate(w.seq_lens)]
    gp = np.arange(0, 2 * spec.batch + 1, 2, dtype=np.int32)
    q_old = W.proxy_query(w.q, cosine, seed=7) if cosine < 1.0 else w.q
    (m, l, o), (out, lse) = _hybrid(w, q_old, old, new, gp)
    (mo, lo, oo), (ref, rlse) = _hybrid_oracle(w, q_old, old, new, gp)
    check_triples(m, l, o, mo, lo, oo, "proxy triples")
    check_out(out, lse, ref, rlse, "proxy merge")
    exact, _ = oracle.attn_full(to_np(w.q), *kv_np(w), w.seq_lens, w.scale)
    err = np.abs(to_np(out) - exact).max()
    if cosine == 1.0:
        assert err <= 2e-3  # exact query everywhere: the hybrid path IS full attention
    else:
        # an approximation: it must differ from exact attention, and by more the worse the proxy
        assert err > 1e-4
        cos = torch.nn.functional.cosine_similarity(q_old.float(), w.q.float(), dim=-1)
        assert (cos - cosine).abs().max().item() < 5e-3
