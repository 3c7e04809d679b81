"""The feedback scheduler policy (paper Algorithm 1) is host-only integer logic; these tests are
its statement, case by case, plus the invariants it must keep (no GPU)."""
import ctypes

import pytest

import paper_2604_18529_amd as hg
from paper_2604_18529_amd import hg_attn as B

POST, PRE = 0, 1


def test_initial_state_is_kmin_and_post_qk():
    st = hg.hg_sched_init(128)
    assert (st.k, st.strategy) == (128, POST)


def test_each_branch_of_the_policy():
    st = hg.hg_sched_init(128)
    # offloaded stage hidden behind the GPU stage: K grows
    assert hg.hg_sched_step(st, 10.0, 6.0, 3.0, 128, 1000, 64) == (192, POST)
    assert hg.hg_sched_step(st, 10.0, 7.0, 3.0, 128, 1000, 64) == (256, POST)  # equality still grows
    # not hidden and K above the threshold: K shrinks, never below K_min
    assert hg.hg_sched_step(st, 10.0, 9.0, 3.0, 128, 1000, 100) == (156, POST)
    assert hg.hg_sched_step(st, 10.0, 9.0, 3.0, 128, 1000, 100) == (128, POST)
    # not hidden and K at the threshold: switch to Pre-QK^T, K stays
    assert hg.hg_sched_step(st, 10.0, 9.0, 3.0, 128, 1000, 100) == (128, PRE)
    # as soon as the stage fits again the tick is Post-QK^T and K grows
    assert hg.hg_sched_step(st, 10.0, 1.0, 1.0, 128, 1000, 100) == (228, POST)
    # growth stops at the number of tokens available
    for _ in range(20):
        hg.hg_sched_step(st, 10.0, 1.0, 1.0, 128, 1000, 100)
    assert (st.k, st.strategy) == (1000, POST)


def test_k_stays_inside_bounds_and_converges_on_a_latency_model():
    """With t_cpu = a + b*K the policy must hover around the largest K that still hides the
    offloaded stage, and never leave [k_min, k_max]."""
    k_min, k_max, step = 128, 8192, 32
    st = hg.hg_sched_init(k_min)
    a, b, t_tx, t_gpu = 0.5, 0.001, 0.3, 3.0
    k_star = (t_gpu - t_tx - a) / b  # 2200
    seen = []
    for _ in range(400):
        k, s = hg.hg_sched_step(st, t_gpu, a + b * st.k, t_tx, k_min, k_max, step)
        assert k_min <= k <= k_max and s in (POST, PRE)
        seen.append(k)
    assert all(abs(k - k_star) <= 2 * step for k in seen[-50:])
    # an executor that is too slow even at k_min ends in Pre-QK^T with K = k_min
    st = hg.hg_sched_init(k_min)
    for _ in range(10):
        k, s = hg.hg_sched_step(st, 1.0, 5.0, 0.1, k_min, k_max, step)
    assert (k, s) == (k_min, PRE)


def test_out_of_range_state_is_clamped_and_bad_arguments_rejected():
    st = B.HgSchedState(5, POST)
    assert hg.hg_sched_step(st, 1.0, 5.0, 0.0, 128, 256, 16) == (128, PRE)
    st = B.HgSchedState(10 ** 6, POST)
    assert hg.hg_sched_step(st, 1.0, 5.0, 0.0, 128, 256, 16) == (240, POST)
    lib = B.load_library()
    ok = B.HgSchedState(128, POST)
    for args in [(1.0, 1.0, 1.0, 0, 10, 1), (1.0, 1.0, 1.0, 10, 5, 1), (1.0, 1.0, 1.0, 10, 20, 0),
                 (float("nan"), 1.0, 1.0, 10, 20, 1), (1.0, -1.0, 1.0, 10, 20, 1), (1.0, float("inf"), 1.0, 10, 20, 1)]:
        assert lib.hg_sched_step(ctypes.byref(ok), *args) == -2
    assert lib.hg_sched_step(None, 1.0, 1.0, 1.0, 10, 20, 1) == -1
    assert lib.hg_sched_init(None, 10) == -1 and lib.hg_sched_init(ctypes.byref(ok), 0) == -2
