"""Shared helpers for the GPU parity tests: run the HIP path through the binding, run the oracle
on the same bits, and compare to the stated bars.

Bars (fp16/fp32 storage, fp32 accumulation; the benchmark spec's tolerance is 2e-3 max-abs on outputs):
  out            max |gpu - oracle| <= 2e-3
  triples        a triple is only defined up to (m, l, O) ~ (m', l e^{m-m'}, O e^{m-m'}); the ABI
                 fixes m as the true maximum, so m is compared directly (1e-3), and l, O through
                 lse = m + log l (1e-3) and O / l (2e-3).
  empty ranges   exactly (-inf, 0, 0).
"""
import numpy as np
import torch

import oracle
import paper_2604_18529_amd as hg

OUT_TOL = 2e-3
M_TOL = 1e-3
LSE_TOL = 1e-3


def to_np(t: torch.Tensor) -> np.ndarray:
    """Host copy as numpy; bfloat16 tensors come back as their uint16 bit patterns, which is how
    the oracle takes that storage type."""
    t = t.detach().cpu()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def kv_np(w):
    """K, V of a workload as numpy arrays that keep the layout (views of the host copies)."""
    k, v = w.k, w.v
    if k.is_contiguous():
        return to_np(k), to_np(v)
    # strided view (token-major storage): copy the storage, rebuild the view
    ks = k.permute(0, 2, 1, 3)
    vs = v.permute(0, 2, 1, 3)
    assert ks.is_contiguous()
    return to_np(ks).transpose(0, 2, 1, 3), to_np(vs).transpose(0, 2, 1, 3)


def check_triples(m_g, l_g, o_g, m_o, l_o, o_o, what=""):
    m_g, l_g, o_g = (to_np(x).astype(np.float64) for x in (m_g, l_g, o_g))
    empty = l_o == 0
    assert np.array_equal(l_g == 0, empty), what + ": empty ranges differ"
    assert np.all(np.isneginf(m_g[empty])) and not o_g[empty].any(), what + ": empty triple is not (-inf, 0, 0)"
    ne = ~empty
    if not ne.any():
        return
    assert np.isfinite(m_g[ne]).all() and np.isfinite(l_g[ne]).all() and np.isfinite(o_g[ne]).all(), what
    dm = np.abs(m_g[ne] - m_o[ne]).max()
    dlse = np.abs((m_g[ne] + np.log(l_g[ne])) - (m_o[ne] + np.log(l_o[ne]))).max()
    dout = np.abs(o_g[ne] / l_g[ne][:, None] - o_o[ne] / l_o[ne][:, None]).max()
    assert dm <= M_TOL, "%s: max |m| error %.3g" % (what, dm)
    assert dlse <= LSE_TOL, "%s: max |lse| error %.3g" % (what, dlse)
    assert dout <= OUT_TOL, "%s: max |O/l| error %.3g" % (what, dout)


def check_out(out_g, lse_g, out_o, lse_o, what=""):
    out_g = to_np(out_g).astype(np.float64)
    assert np.isfinite(out_g).all(), what
    d = np.abs(out_g - out_o).max() if out_o.size else 0.0
    assert d <= OUT_TOL, "%s: max |out| error %.3g" % (what, d)
    if lse_g is not None:
        lse_g = to_np(lse_g).astype(np.float64)
        fin = np.isfinite(lse_o)
        assert np.array_equal(np.isneginf(lse_g), ~fin), what + ": -inf lse pattern differs"
        if fin.any():
            dl = np.abs(lse_g[fin] - lse_o[fin]).max()
            assert dl <= LSE_TOL, "%s: max |lse| error %.3g" % (what, dl)


def run_all_and_check(w, ranges=None, group_ptr=None, what=""):
    """partial + merge + full on the GPU against the oracle, for workload w."""
    ranges = w.ranges if ranges is None else ranges
    group_ptr = w.group_ptr if group_ptr is None else group_ptr
    kn, vn = kv_np(w)
    qn = to_np(w.q)
    m, l, o = hg.hg_attn_partial(w.q, w.k, w.v, w.seq_lens, ranges, w.scale)
    mo, lo, oo = oracle.attn_partial(qn, kn, vn, w.seq_lens, w.scale, ranges)
    check_triples(m, l, o, mo, lo, oo, what + " partial")
    out, lse = hg.hg_attn_merge(m, l, o, group_ptr)
    ref, rlse = oracle.attn_merge(mo, lo, oo, group_ptr)
    check_out(out, lse, ref, rlse, what + " merge")
    fout, flse = hg.hg_attn_full(w.q, w.k, w.v, w.seq_lens, w.scale)
    fref, frlse = oracle.attn_full(qn, kn, vn, w.seq_lens, w.scale)
    check_out(fout, flse, fref, frlse, what + " full")
    torch.cuda.synchronize()
    return (m, l, o), (out, lse), (fout, flse)
