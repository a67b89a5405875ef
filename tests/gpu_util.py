"""Helpers that run the HIP path through the binding and bring results back as numpy."""
from __future__ import annotations

import numpy as np
import torch

import paper_2602_22575_amd as s2o


def to_dev(bits: np.ndarray, dev="cuda:0"):
    return torch.from_numpy(bits.view(np.int16)).to(dev).view(torch.bfloat16)


def params_for(w, **kw):
    return s2o.make_params(w.Z, w.H, w.Hkv, w.L, w.D, w.S, w.BM, w.BN, **kw)


def bits_of(t: torch.Tensor) -> np.ndarray:
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def gpu_plan(w, Qd, Kd, non_causal=0):
    p = params_for(w, non_causal=non_causal)
    out = s2o.s2o_plan(Qd, Kd, p, want_scores=True)
    torch.cuda.synchronize()
    assert int(out.status.item()) == 0, f"plan status {int(out.status.item())} (S2O_PLAN_* bits)"
    return out, {k: getattr(out, k).cpu().numpy() for k in ("q_perm", "kv_perm", "s_q", "s_k", "q_mean", "k_guide")}


def gpu_attention(w, Qd, Kd, Vd, q_perm, kv_perm, tau, stop_mode=0, use_q_perm=1, two_pass=True, max_tiles=0,
                  non_causal=0):
    p = params_for(w, stop_mode=stop_mode, use_q_perm=use_q_perm, max_prefix_tiles=max_tiles,
                   non_causal=non_causal)
    O, c, s = s2o.s2o_attention(Qd, Kd, Vd, p, q_perm, kv_perm, tau, two_pass=two_pass)
    torch.cuda.synchronize()
    return bits_of(O), c.cpu().numpy(), s.cpu().numpy()
