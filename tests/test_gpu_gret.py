"""Parity of gated retention (section 3.1, Eq. 4-7) on the GPU with the fp64
oracle: the recurrent kernel (prefill of the shapes without a chunkwise path,
and the decode step), the chunkwise MFMA path, carried states, and the fused
GroupNorm. Tolerances: fp32 1e-4; bf16 max-abs 2e-2 and sum-ratio 2e-3 on
GroupNorm'ed outputs (unit variance); raw outputs (no GroupNorm) are compared
after dividing both sides by max(1, max|ref|), states likewise."""
import math

import numpy as np
import pytest
import torch

import oracle
import yoco_synth as ys

pytestmark = pytest.mark.gpu

TD = {"f32": torch.float32, "bf16": torch.bfloat16}


@pytest.fixture(scope="module")
def yoco():
    import paper_2405_05254_amd as y
    y.lib()                       # fails loudly if libyoco.so is not built
    assert torch.cuda.is_available()
    return y


def dev(a, dtype):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda").to(TD[dtype])


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def check(got, ref, dtype, what, relative=False):
    unit = max(1.0, float(np.abs(ref).max())) if relative else 1.0
    st = ys.error_stats(got / unit, ref / unit)
    tol = ys.TOL[dtype]
    print("%s: max_abs %.3e mean_rel %.3e (unit %.3g)" % (what, st["max_abs"], st["mean_rel"], unit), flush=True)
    assert np.isfinite(got).all(), what
    assert st["max_abs"] <= tol["max_abs"] and st["mean_rel"] <= tol["mean_rel"], (what, st)


def oracle_gret(q, k, v, lg, scale, group_norm, eps, S0=None):
    """Per sequence: the recurrent form (pinned equal to the parallel definition), then Eq. 7's GroupNorm.
    States in the library's layout [H,dv,dk]."""
    O, S = [], []
    for b in range(q.shape[0]):
        s0 = None if S0 is None else np.transpose(S0[b], (0, 2, 1))
        o, s = oracle.gret_recurrent(q[b], k[b], v[b], np.exp(lg[b].astype(np.float64)), scale, S0=s0)
        O.append(oracle.group_norm_heads(o, eps) if group_norm else o)
        S.append(np.transpose(s, (0, 2, 1)))
    return np.stack(O), np.stack(S)


RECURRENT_CASES = [
    # dtype, B, T, H, dk, dv, group_norm
    ("f32", 1, 512, 4, 64, 64, True),        # the tiny configuration's shape
    ("f32", 2, 77, 3, 32, 64, False),        # dk != dv, raw output
    ("f32", 1, 40, 2, 128, 72, True),        # dv not a multiple of 32
    ("bf16", 2, 300, 3, 128, 128, True),
    ("bf16", 1, 130, 2, 128, 128, False),
    ("bf16", 1, 64, 2, 64, 128, True),
    ("bf16", 1, 1, 2, 128, 128, True),       # a single row
]


@pytest.mark.parametrize("dtype,B,T,H,dk,dv,gn", RECURRENT_CASES)
def test_gret_prefill_recurrent_path_matches_oracle(yoco, dtype, B, T, H, dk, dv, gn):
    scale = 1.0 / math.sqrt(dk)
    q, k, v, lg = ys.gret_inputs(T + dk, B, T, H, dk, dv, 1.0, dtype)
    rng = np.random.default_rng(1)
    S0 = rng.standard_normal((B, H, dv, dk)).astype(np.float32)
    s_in = torch.from_numpy(S0).cuda()
    s_out = torch.full_like(s_in, float("nan"))
    o = yoco.gret_prefill(dev(q, dtype), dev(k, dtype), dev(v, dtype), torch.from_numpy(lg).cuda(), scale, chunk=256,
                          group_norm=gn, eps=1e-6, state_in=s_in, state_out=s_out)
    torch.cuda.synchronize()
    ref_o, ref_s = oracle_gret(q, k, v, lg, scale, gn, 1e-6, S0)
    check(host(o), ref_o, dtype, "gret recurrent path o %s" % ((dtype, B, T, H, dk, dv, gn),), relative=not gn)
    check(host(s_out), ref_s, "f32", "gret recurrent path state", relative=True)


def test_gret_decode_steps_continue_a_prefill(yoco):
    """Prefill of 50 rows, then 30 single-row steps with the state updated in place (different decays per
    sequence and head), against one oracle pass over all 80 rows."""
    B, T0, steps, H, dk, dv = 3, 50, 30, 4, 128, 128
    scale = 1.0 / math.sqrt(dk)
    q, k, v, lg = ys.gret_inputs(7, B, T0 + steps, H, dk, dv, 1.0, "bf16")
    ref_o, ref_s = oracle_gret(q, k, v, lg, scale, True, 1e-6)
    qd, kd, vd, gd = dev(q, "bf16"), dev(k, "bf16"), dev(v, "bf16"), torch.from_numpy(lg).cuda()
    state = torch.zeros(B, H, dv, dk, dtype=torch.float32, device="cuda")
    o0 = yoco.gret_prefill(qd[:, :T0].contiguous(), kd[:, :T0].contiguous(), vd[:, :T0].contiguous(),
                           gd[:, :T0].contiguous(), scale, state_in=None, state_out=state)
    outs = [host(o0)]
    for i in range(T0, T0 + steps):
        o = yoco.gret_decode(qd[:, i].contiguous(), kd[:, i].contiguous(), vd[:, i].contiguous(), gd[:, i].contiguous(),
                             state, scale)
        outs.append(host(o)[:, None])
    torch.cuda.synchronize()
    check(np.concatenate(outs, axis=1), ref_o, "bf16", "gret prefill + decode steps")
    check(host(state), ref_s, "f32", "gret state after the steps", relative=True)


def test_gret_empty_prefill_copies_the_state(yoco):
    B, H, dk, dv = 2, 3, 64, 32
    s_in = torch.randn(B, H, dv, dk, device="cuda")
    s_out = torch.zeros_like(s_in)
    e = torch.empty(B, 0, H, dk, device="cuda")
    yoco.gret_prefill(e, e, torch.empty(B, 0, H, dv, device="cuda"), torch.empty(B, 0, H, device="cuda"), 1.0,
                      state_in=s_in, state_out=s_out)
    assert torch.equal(s_in, s_out)
    yoco.gret_prefill(e, e, torch.empty(B, 0, H, dv, device="cuda"), torch.empty(B, 0, H, device="cuda"), 1.0,
                      state_in=None, state_out=s_out)
    assert torch.count_nonzero(s_out).item() == 0
