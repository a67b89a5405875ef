"""s2o_plan_static -- the ranking for callers that cannot allocate device memory (its scratch is
an array built into the library) -- against s2o_plan on the same inputs, through the C ABI."""
import ctypes as C

import numpy as np
import pytest

from paper_2602_22575_amd import binding as b, inputs
import gpu_util as gu

pytestmark = pytest.mark.gpu


def _both(w):
    import torch
    Qb, Kb, _ = inputs.make_qkv(w)
    Qd, Kd = gu.to_dev(Qb), gu.to_dev(Kb)
    p = gu.params_for(w)
    assert b.s2o_plan_sizes(p)["scratch"] <= b.STATIC_SCRATCH_BYTES
    ref = b.s2o_plan(Qd, Kd, p, want_scores=True)
    got = b.s2o_plan(Qd, Kd, p, want_scores=True, static_scratch=True)
    torch.cuda.synchronize()
    return ref, got


def _assert_same(ref, got):
    import torch
    assert int(ref.status.item()) == 0 and int(got.status.item()) == 0
    for name in ("q_perm", "kv_perm", "s_q", "s_k", "q_mean", "k_guide"):
        a_, b_ = getattr(ref, name), getattr(got, name)
        assert a_.shape == b_.shape and torch.equal(a_.view(torch.int32), b_.view(torch.int32)), name


def test_static_scratch_plan_equals_the_caller_scratch_plan(gpu):
    """Two calls in a row on the shared built-in array, the second on a smaller input: maps and
    scores must equal s2o_plan's bit for bit both times (integer outputs exact; the scores come
    from the same kernels in the same order, so they are compared as bits too)."""
    print("case: s2o_plan_static, Llama head shape at 8K", flush=True)
    big = inputs.workload("llama8k")
    _assert_same(*_both(big))
    print("case: s2o_plan_static again, smaller input (L=1024, 4 heads)", flush=True)
    small = inputs.workload("llama8k", L=1024, S=256, H=4, Hkv=2, seed=17)
    _assert_same(*_both(small))
    # and once more on the first shape: nothing left over from the smaller call may leak in
    print("case: s2o_plan_static, first shape again", flush=True)
    _assert_same(*_both(big))


def test_static_scratch_refuses_what_does_not_fit(gpu):
    lib = b.load_library()
    p = b.make_params(1, 32, 8, 131072, 128, 2048)
    assert b.s2o_plan_sizes(p)["scratch"] > b.STATIC_SCRATCH_BYTES
    out = b.S2OPlanOut(0x1000, 0x1000, None, None, None, None, None)
    fake = C.c_void_p(0x10000)
    assert lib.s2o_plan_static(fake, fake, C.byref(p), C.byref(out), None) == b.S2O_ESCRATCH
