"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
the header declares, answers size queries and rejects bad arguments before touching HIP."""
import ctypes as C
import os
import re

import pytest

from paper_2602_22575_amd import binding as b

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return b.load_library()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "s2o.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(s2o_[a-z_]+)\s*\(", header))
    assert declared == set(b.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None
    assert lib.s2o_version() == 4


def test_struct_layout_matches_header(lib):
    assert C.sizeof(b.S2OParams) == 14 * 4 + 12 * 8
    assert C.sizeof(b.S2OPlanOut) == 7 * 8


def test_size_queries():
    p = b.make_params(1, 32, 8, 131072, 128, 2048)
    sz = b.s2o_plan_sizes(p)
    N, S = 64, 2048
    P = S * N * (N - 1) // 2
    assert sz["q_perm"] == 32 * 131072 * 4 and sz["s_q"] == sz["q_perm"]
    assert sz["kv_perm"] == 32 * P * 4 and sz["s_k"] == sz["kv_perm"]
    assert sz["q_mean"] == 32 * N * 128 * 4 and sz["k_guide"] == 8 * 128 * 4
    assert sz["scratch"] >= 32 * P * 8 and sz["scratch"] % 256 == 0
    asz = b.s2o_attention_sizes(p)
    assert asz["counts"] == 32 * (131072 // 64) * 4
    assert asz["scratch"] == 32 * 131072 * (128 + 2) * 4      # fp32 acc, l, m per query row
    # non-causal setting: rows of L ranked keys for every segment, no state buffer
    pn = b.make_params(1, 32, 8, 131072, 128, 2048, non_causal=1)
    szn = b.s2o_plan_sizes(pn)
    assert szn["kv_perm"] == 32 * N * 131072 * 4 and szn["s_k"] == szn["kv_perm"]
    assert szn["q_perm"] == sz["q_perm"] and szn["scratch"] >= 32 * N * 131072 * 8
    assert b.s2o_attention_sizes(pn)["scratch"] == 0


@pytest.mark.parametrize("kw,code", [
    (dict(L=1000), b.S2O_EINVAL),                 # L % S != 0
    (dict(H=6, Hkv=4), b.S2O_EINVAL),             # H % Hkv != 0
    (dict(Z=0), b.S2O_EINVAL),
    (dict(D=64), b.S2O_EUNSUPPORTED),
    (dict(BM=32), b.S2O_EUNSUPPORTED),
    (dict(BM=128, S=192, L=768), b.S2O_EUNSUPPORTED),   # S % B_M != 0
    (dict(BN=128), b.S2O_EUNSUPPORTED),
    (dict(S=96, L=960), b.S2O_EUNSUPPORTED),      # S % 64 != 0
    (dict(S=16384, L=32768), b.S2O_EUNSUPPORTED),
    (dict(stop_mode=3), b.S2O_EINVAL),
    (dict(max_prefix_tiles=-1), b.S2O_EINVAL),
    (dict(non_causal=2), b.S2O_EINVAL),
    (dict(use_q_perm=5), b.S2O_EINVAL),
    (dict(softmax_scale=-1.0), b.S2O_EINVAL),
    (dict(q_stride=(0, 0, 100)), b.S2O_EINVAL),   # row stride not 16-byte aligned / < D
    (dict(L=2 << 20, S=2048), b.S2O_EUNSUPPORTED),          # plan: a row's sample no longer fits the LDS sort
    (dict(k_stride=(1 << 40, 1 << 36, 1 << 23)), b.S2O_EUNSUPPORTED),   # a K row stride of 16 MiB
    (dict(L=1 << 20, S=2048, v_stride=(1 << 40, 1 << 36, 4096)), b.S2O_EUNSUPPORTED),   # a V head beyond 4 GiB
])
def test_bad_params_are_rejected(kw, code):
    base = dict(Z=1, H=4, Hkv=2, L=1024, D=128, S=256)
    base.update(kw)
    with pytest.raises(b.S2OError) as e:
        b.s2o_plan_sizes(b.make_params(**base))
    assert e.value.code == code


def test_plan_status_bits_are_declared():
    """The status word of s2o_plan_out and its bits exist in the header and in the binding."""
    header = open(os.path.join(ROOT, "include", "s2o.h")).read()
    for name, bit in (("S2O_PLAN_STAGE_OVERFLOW", 1), ("S2O_PLAN_COUNT_MISMATCH", 2), ("S2O_PLAN_SPAN_OVERFLOW", 4),
                      ("S2O_PLAN_BAD_RANK", 8)):
        assert re.search(rf"{name}\s*=\s*{bit}\b", header), name
    assert re.search(r"int32_t\*\s*status;", header)
    assert [f[0] for f in b.S2OPlanOut._fields_][-1] == "status"


def test_segment_length_limit_applies_to_the_plan_only():
    """The ranking sorts a segment's query scores in LDS (S <= 8192); attention takes any S
    (S = L is dense contiguous causal attention, the appendix's kernel A)."""
    p = b.make_params(1, 4, 2, 32768, 128, 32768)
    assert b.s2o_attention_sizes(p)["scratch"] == 4 * 32768 * 130 * 4
    with pytest.raises(b.S2OError) as e:
        b.s2o_plan_sizes(p)
    assert e.value.code == b.S2O_EUNSUPPORTED


def test_null_and_scratch_errors_come_before_any_hip_call(lib):
    p = b.make_params(1, 4, 2, 1024, 128, 256)
    out = b.S2OPlanOut(0x1000, 0x1000, None, None, None, None)
    fake = C.c_void_p(0x10000)
    assert lib.s2o_plan(None, fake, C.byref(p), C.byref(out), fake, 1 << 40, None) == b.S2O_EINVAL
    assert lib.s2o_plan(fake, fake, None, C.byref(out), fake, 1 << 40, None) == b.S2O_EINVAL
    assert lib.s2o_plan(fake, fake, C.byref(p), None, fake, 1 << 40, None) == b.S2O_EINVAL
    assert lib.s2o_plan(fake, fake, C.byref(p), C.byref(out), None, 1 << 40, None) == b.S2O_ESCRATCH
    assert lib.s2o_plan(fake, fake, C.byref(p), C.byref(out), fake, 16, None) == b.S2O_ESCRATCH
    assert lib.s2o_plan(fake, fake, C.byref(p), C.byref(out), C.c_void_p(0x10010), 1 << 40, None) == b.S2O_ESCRATCH
    no_qperm = b.S2OPlanOut(None, 0x1000, None, None, None, None)
    assert lib.s2o_plan(fake, fake, C.byref(p), C.byref(no_qperm), fake, 1 << 40, None) == b.S2O_EINVAL
    assert lib.s2o_plan(C.c_void_p(0x10002), fake, C.byref(p), C.byref(out), fake, 1 << 40, None) == b.S2O_EINVAL
    # attention
    args = [fake, fake, fake, C.byref(p), fake, fake, C.c_float(0.0), fake, None, None, None, 0, None]
    for i in (0, 1, 2, 7):
        bad = list(args)
        bad[i] = None
        assert lib.s2o_attention(*bad) == b.S2O_EINVAL
    bad = list(args); bad[4] = None                    # q_perm missing while use_q_perm = 1
    assert lib.s2o_attention(*bad) == b.S2O_EINVAL
    bad = list(args); bad[5] = None                    # kv_perm missing while N > 1
    assert lib.s2o_attention(*bad) == b.S2O_EINVAL
    bad = list(args); bad[6] = C.c_float(float("nan"))
    assert lib.s2o_attention(*bad) == b.S2O_EINVAL
    bad = list(args); bad[10] = fake; bad[11] = 4096   # two-pass state buffer too small
    assert lib.s2o_attention(*bad) == b.S2O_ESCRATCH
    bad = list(args); bad[10] = C.c_void_p(0x10010); bad[11] = 1 << 40
    assert lib.s2o_attention(*bad) == b.S2O_ESCRATCH
    # non-causal setting: no own-segment pass, the threshold must be finite
    pn = b.make_params(1, 4, 2, 1024, 128, 256, non_causal=1)
    assert lib.s2o_attention_local(fake, fake, fake, C.byref(pn), fake, 1 << 40, None) == b.S2O_EUNSUPPORTED
    nargs = list(args); nargs[3] = C.byref(pn)
    bad = list(nargs); bad[6] = C.c_float(float("inf"))
    assert lib.s2o_attention(*bad) == b.S2O_EINVAL
    bad = list(nargs); bad[5] = C.c_void_p(0x10004)    # a map, but misaligned
    assert lib.s2o_attention(*bad) == b.S2O_EINVAL
    p.struct_size = 8
    assert lib.s2o_attention(*args) == b.S2O_EINVAL
    assert lib.s2o_strerror(b.S2O_ESCRATCH).decode().startswith("scratch")


def test_inputs_are_deterministic_and_bf16():
    import numpy as np
    from paper_2602_22575_amd import inputs
    w = inputs.workload("tiny")
    a = inputs.make_qkv(w)
    c = inputs.make_qkv(w)
    for x, y in zip(a, c):
        assert x.dtype == np.uint16 and np.array_equal(x, y)
    assert a[0].shape == (1, 1, 2048, 128) and a[1].shape == (1, 1, 2048, 128)
    v = inputs.bf16_bits_to_f32(a[2]).astype(np.float64)
    assert abs(v.mean()) < 0.01 and abs(v.std() - 1) < 0.01
    w2 = inputs.workload("llama8k", L=1024, S=256)
    q, k, _ = inputs.make_qkv(w2)
    assert q.shape == (1, 32, 1024, 128) and k.shape == (1, 8, 1024, 128)
    assert inputs.heavy_positions(w2, 0, 3)[:4].tolist() == [0, 1, 2, 3]
