"""Parity of gated retention (section 3.1, Eq. 4-7) on the GPU with the fp64
oracle: the recurrent kernel (prefill of the shapes without a chunkwise path,
and the decode step), the chunkwise MFMA path, carried states, and the fused
GroupNorm. Tolerances: fp32 1e-4; bf16 max-abs 2e-2 and sum-ratio 2e-3 on
GroupNorm'ed outputs (unit variance); raw outputs (no GroupNorm) are compared
after dividing both sides by max(1, max|ref|), states likewise (fp32 bound for
the recurrent kernel's states, a tenth of the bf16 bound for the chunkwise
path's, whose products run on fp16 operands)."""
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


# The chunkwise path forms its states from V * decay rounded to fp16 (11 significant bits, 2.4e-4 relative per
# term) on the matrix cores with fp32 accumulation: its states are held to a tenth of the bf16 output bound.
STATE_F16 = dict(max_abs=2e-3, mean_rel=1e-3)


def check(got, ref, dtype, what, relative=False):
    unit = max(1.0, float(np.abs(ref).max())) if relative else 1.0
    st = ys.error_stats(got / unit, ref / unit)
    tol = STATE_F16 if dtype == "state_f16" else ys.TOL[dtype]
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


# ------------------------------------------------ chunkwise path on the matrix cores (Eq. 6)
CHUNK_CASES = [
    # B, T, H, chunk, group_norm, mean of -ln(gamma), carry a state in
    (1, 700, 2, 256, True, 0.04, True),        # two whole chunks and a ragged one; several tiles with a ragged tail
    (2, 1024, 3, 128, True, 0.04, False),      # chunk = one query block
    (1, 1300, 2, 512, False, 0.04, True),      # raw output
    (1, 1100, 1, 1024, True, 0.01, True),      # the largest chunk
    (1, 100, 2, 256, True, 0.04, True),        # shorter than a chunk and than a query block
    (1, 129, 2, 256, True, 0.04, False),       # one row into the second query block
    (1, 640, 2, 256, True, 0.5, True),         # strong decay: gamma around 0.6, 2^-190 across a chunk
    (1, 640, 2, 256, False, 0.0005, True),     # almost no decay: long memory, large states
]


def test_gret_chunkwise_large_magnitudes(yoco):
    """Inputs of standard deviation 4 (scores of magnitude ~100 before the scale, states in the thousands):
    far from the fp16 limits of the chunkwise path, results still within the bounds."""
    B, T, H, d, chunk = 1, 700, 2, 128, 256
    scale = 1.0 / math.sqrt(d)
    q, k, v, lg = ys.gret_inputs(31, B, T, H, d, d, 4.0, "bf16")
    ws = torch.empty(yoco.gret_prefill_workspace(B, T, H, d, d, chunk, yoco.BF16), dtype=torch.uint8, device="cuda")
    s_out = torch.empty(B, H, d, d, dtype=torch.float32, device="cuda")
    for gn in (True, False):
        o = yoco.gret_prefill(dev(q, "bf16"), dev(k, "bf16"), dev(v, "bf16"), torch.from_numpy(lg).cuda(), scale, chunk=chunk,
                              group_norm=gn, state_out=s_out, workspace=ws)
        torch.cuda.synchronize()
        ref_o, ref_s = oracle_gret(q, k, v, lg, scale, gn, 1e-6)
        check(host(o), ref_o, "bf16", "gret chunkwise, std 4, group_norm=%s" % gn, relative=not gn)
    check(host(s_out), ref_s, "state_f16", "gret chunkwise, std 4: state", relative=True)


@pytest.mark.parametrize("B,T,H,chunk,gn,mld,carry", CHUNK_CASES)
def test_gret_prefill_chunkwise_matches_oracle(yoco, B, T, H, chunk, gn, mld, carry):
    d = 128
    scale = 1.0 / math.sqrt(d)
    q, k, v, lg = ys.gret_inputs(T + chunk, B, T, H, d, d, 1.0, "bf16", mean_log_decay=mld)
    rng = np.random.default_rng(2)
    S0 = rng.standard_normal((B, H, d, d)).astype(np.float32) if carry else None
    s_in = torch.from_numpy(S0).cuda() if carry else None
    s_out = torch.full((B, H, d, d), float("nan"), dtype=torch.float32, device="cuda")
    nbytes = yoco.gret_prefill_workspace(B, T, H, d, d, chunk, yoco.BF16)
    assert nbytes > 0
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    args = (dev(q, "bf16"), dev(k, "bf16"), dev(v, "bf16"), torch.from_numpy(lg).cuda(), scale)
    o = yoco.gret_prefill(*args, chunk=chunk, group_norm=gn, eps=1e-6, state_in=s_in, state_out=s_out, workspace=ws)
    torch.cuda.synchronize()
    ref_o, ref_s = oracle_gret(q, k, v, lg, scale, gn, 1e-6, S0)
    what = "gret chunkwise %s" % ((B, T, H, chunk, gn, mld, carry),)
    check(host(o), ref_o, "bf16", what + " o", relative=not gn)
    check(host(s_out), ref_s, "state_f16", what + " state", relative=True)
    # the recurrent kernel on the same inputs (no workspace): both paths are the same function
    s_rec = torch.empty_like(s_out)
    o_rec = yoco.gret_prefill(*args, chunk=chunk, group_norm=gn, eps=1e-6, state_in=s_in, state_out=s_rec)
    check(host(o), host(o_rec), "bf16", what + " against the recurrent kernel", relative=not gn)


def test_gret_chunkwise_split_prompt_carries_the_state(yoco):
    """A prompt processed as 384 + 516 rows with the state handed over equals one call over 900 rows."""
    B, T, H, d, chunk = 1, 900, 2, 128, 256
    scale = 1.0 / math.sqrt(d)
    q, k, v, lg = ys.gret_inputs(11, B, T, H, d, d, 1.0, "bf16")
    ws = torch.empty(yoco.gret_prefill_workspace(B, T, H, d, d, chunk, yoco.BF16), dtype=torch.uint8, device="cuda")
    qd, kd, vd, gd = dev(q, "bf16"), dev(k, "bf16"), dev(v, "bf16"), torch.from_numpy(lg).cuda()
    state = torch.empty(B, H, d, d, dtype=torch.float32, device="cuda")
    o1 = yoco.gret_prefill(qd[:, :384].contiguous(), kd[:, :384].contiguous(), vd[:, :384].contiguous(),
                           gd[:, :384].contiguous(), scale, chunk=chunk, state_in=None, state_out=state, workspace=ws)
    o2 = yoco.gret_prefill(qd[:, 384:].contiguous(), kd[:, 384:].contiguous(), vd[:, 384:].contiguous(),
                           gd[:, 384:].contiguous(), scale, chunk=chunk, state_in=state, state_out=state, workspace=ws)
    torch.cuda.synchronize()
    ref_o, ref_s = oracle_gret(q, k, v, lg, scale, True, 1e-6)
    check(np.concatenate([host(o1), host(o2)], axis=1), ref_o, "bf16", "gret chunkwise, split prompt")
    check(host(state), ref_s, "state_f16", "gret chunkwise, split prompt: state", relative=True)


def test_gret_prefill_without_enough_workspace_uses_the_recurrence(yoco):
    B, T, H, d = 1, 300, 2, 128
    q, k, v, lg = ys.gret_inputs(12, B, T, H, d, d, 1.0, "bf16")
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    o = yoco.gret_prefill(dev(q, "bf16"), dev(k, "bf16"), dev(v, "bf16"), torch.from_numpy(lg).cuda(), 0.1, chunk=256,
                          workspace=small)
    torch.cuda.synchronize()
    ref_o, _ = oracle_gret(q, k, v, lg, 0.1, True, 1e-6)
    check(host(o), ref_o, "bf16", "gret with a workspace that is too small")
    assert yoco.gret_prefill_workspace(B, T, H, 64, d, 256, yoco.BF16) == 0         # no chunkwise path for dk = 64
    assert yoco.gret_prefill_workspace(B, T, H, d, d, 192, yoco.BF16) == 0          # nor for a chunk that is not n * 128


@pytest.mark.parametrize("dtype,T,chunked", [("bf16", 600, True), ("bf16", 200, False), ("f32", 90, False)])
def test_gret_fused_swish_gate(yoco, dtype, T, chunked):
    """Eq. 7 without W_O in one call: swish(gate) * GroupNorm(gRet), on both paths and in the decode step."""
    B, H, d = 1, 2, 128 if dtype == "bf16" else 64
    scale = 1.0 / math.sqrt(d)
    q, k, v, lg = ys.gret_inputs(41 + T, B, T + 1, H, d, d, 1.0, dtype)
    gate = ys.normal(np.random.default_rng(T), (B, T + 1, H, d), 1.5, dtype)
    ref_o, _ = oracle_gret(q, k, v, lg, scale, True, 1e-6)
    ref = oracle.swish(gate) * ref_o
    ws = None
    if chunked:
        ws = torch.empty(yoco.gret_prefill_workspace(B, T, H, d, d, 256, yoco.BF16), dtype=torch.uint8, device="cuda")
    state = torch.empty(B, H, d, d, dtype=torch.float32, device="cuda")
    cut = lambda a: dev(a[:, :T], dtype).contiguous()
    o = yoco.gret_prefill(cut(q), cut(k), cut(v), torch.from_numpy(lg[:, :T].copy()).cuda(), scale, chunk=256, state_out=state,
                          workspace=ws, gate=cut(gate))
    last = lambda a: dev(a[:, T], dtype).contiguous()
    od = yoco.gret_decode(last(q), last(k), last(v), torch.from_numpy(lg[:, T].copy()).cuda(), state, scale, gate=last(gate))
    torch.cuda.synchronize()
    # gated outputs are not unit-variance any more (|swish(g)| reaches ~6 here): compared relative to the largest one
    check(host(o), ref[:, :T], dtype, "gret with the fused gate, prefill (%s)" % ("chunkwise" if chunked else "recurrent"),
          relative=True)
    check(host(od), ref[:, T], dtype, "gret with the fused gate, decode step", relative=True)


def test_gret_prefill_full_size_sampled(yoco):
    """The benchmark's gated-retention launch (T = 32768, 24 heads x 128, chunk 256, GroupNorm), three heads
    checked row by row against the oracle's recurrence, and the final state of those heads."""
    B, T, H, d, chunk = 1, 32768, 24, 128, 256
    scale = 1.0 / math.sqrt(d)
    q, k, v, lg = ys.gret_inputs(0, B, T, H, d, d, 1.0, "bf16")
    ws = torch.empty(yoco.gret_prefill_workspace(B, T, H, d, d, chunk, yoco.BF16), dtype=torch.uint8, device="cuda")
    s_out = torch.empty(B, H, d, d, dtype=torch.float32, device="cuda")
    o = yoco.gret_prefill(dev(q, "bf16"), dev(k, "bf16"), dev(v, "bf16"), torch.from_numpy(lg).cuda(), scale, chunk=chunk,
                          state_out=s_out, workspace=ws)
    torch.cuda.synchronize()
    got, gs = host(o), host(s_out)
    for h in (0, 11, 23):
        ref_o, ref_s = oracle_gret(q[:, :, h:h + 1], k[:, :, h:h + 1], v[:, :, h:h + 1], lg[:, :, h:h + 1], scale, True, 1e-6)
        check(got[:, :, h:h + 1], ref_o, "bf16", "gret full size, head %d" % h)
        check(gs[:, h:h + 1], ref_s, "state_f16", "gret full size, state of head %d" % h, relative=True)


# ------------------------------------------------ the stack with a gated-retention self-decoder
def test_tiny_gret_stack_matches_oracle(yoco):
    """Tiny fp32 stack whose self-decoder is multi-head gated retention (Eq. 7): full forward against the
    oracle, early exit against the full forward, and prompt + teacher-forced decode steps (recurrent state
    carried from the prefill) against the oracle's all-at-once logits."""
    from paper_2405_05254_amd.stack import YocoStack
    c = ys.CONFIGS["tiny_fp32"]
    spec = dict(c["stack"], self_kind="gret", tau=16.0)
    w = ys.stack_weights(c["seed"], spec, "f32")
    T0, steps = 300, 30
    tok = ys.tokens(c["seed"] + 3, T0 + steps, spec["vocab"])
    ref = oracle.yoco_stack(tok, w, "full")
    st = YocoStack(w, torch.float32)
    t = torch.from_numpy(tok).cuda()
    full = host(st.forward_full(t))
    ee = host(st.forward_early_exit(t)[0])
    print("gret stack: full vs oracle %.3e, early exit vs full %.3e" % (np.abs(full - ref).max(), np.abs(ee[0] - full[-1]).max()),
          flush=True)
    assert np.abs(full - ref).max() <= 1e-3
    assert np.abs(ee[0] - full[-1]).max() <= 1e-3
    state = st.new_generation_state(T0 + steps)
    logits = [host(st.prefill(t[:T0], state))[0]]
    for i in range(steps):
        logits.append(host(st.decode_step(t[T0 + i], state))[0])
    err = np.abs(np.stack(logits) - ref[T0 - 1:]).max()
    print("gret stack: prefill + %d decode steps vs oracle %.3e" % (steps, err), flush=True)
    assert err <= 1e-3


def test_bf16_gret_stack_early_exit_and_generation(yoco):
    """The end-to-end architecture with a gated-retention self-decoder (d_model 2048, 16 x 128 heads, reduced to
    3 + 3 layers) at T = 3000, bf16: the chunkwise MFMA path in the prefill. Three checks:
    (1) early exit against the GPU full forward (Fig. 3: same kernels on both sides, 1e-3);
    (2) at the attention boundary, layer by layer and teacher-forced: the chunkwise prefill of the first T - 8 rows
        followed by 8 recurrent decode steps, fed the full forward's own q, k, v, decays and gates of that layer,
        must reproduce the full forward's attention outputs of the last 8 rows to the bf16 bounds (both sides round
        the same fp32 value once; the carried state differs by the chunkwise path's fp16-operand rounding);
    (3) free-running: a prompt + 8 decode steps against the full forward's logits. Here a rounding that falls
        differently in one layer changes the inputs of the next, whose bf16 roundings (q, k, v, gate, o: ulp 2^-8)
        then flip with a probability that grows with the incoming difference: a random walk over about 6 layers x 5
        rounded tensors of steps of about 2e-3 of the values' scale, i.e. about sqrt(30) * 2e-3 = 1.1e-2 of the logit
        scale in the worst of the 9 x 4096 logits compared (measured 1-2 %). The bound is 5 % of the largest logit:
        a check against gross errors (a wrong state hand-over, a missed row costs far more); the fp32 stack above
        pins the same flow to 1e-3 absolute against the oracle, and (2) holds the kernels to the bf16 bounds."""
    from paper_2405_05254_amd.stack import YocoStack
    import paper_2405_05254_amd as yb
    c = ys.CONFIGS["e2e_early_exit_128k"]
    s = dict(c["stack"], n_self=3, n_cross=3, vocab=4096, self_kind="gret", tau=16.0)
    T = 3000
    w = ys.stack_weights(c["seed"], s, "bf16")
    tok = torch.from_numpy(ys.tokens(c["seed"], T, s["vocab"])).cuda()
    st = YocoStack(w, torch.bfloat16)
    st.capture = {"self%d" % n: None for n in range(3)}
    full = host(st.forward_full(tok, rows=slice(T - 9, T)))
    caps = dict(st.capture)
    st.capture = None
    ee = host(st.forward_early_exit(tok)[0])
    err = np.abs(ee - full[-1:]).max()
    print("bf16 gret stack early-exit vs full: %.3e (logit scale %.3f)" % (err, np.abs(full).max()), flush=True)
    assert err <= 1e-3
    # (2) the attention boundary, teacher-forced
    H, d, Tp = st.Hq, st.d, T - 8
    for n in range(3):
        q, k, v, o, lg, gate = caps["self%d" % n]
        state = torch.zeros(1, H, d, d, dtype=torch.float32, device="cuda")
        nbytes = yb.gret_prefill_workspace(1, Tp, H, d, d, 256, yb.BF16)
        assert nbytes > 0                                    # the chunkwise path, not the recurrence
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        o_pre = yb.gret_prefill(q[None, :Tp].contiguous(), k[None, :Tp].contiguous(), v[None, :Tp].contiguous(),
                                lg[None, :Tp].contiguous(), st.scale, chunk=256, group_norm=True, eps=st.eps, state_out=state,
                                workspace=ws, gate=gate[None, :Tp].contiguous())
        assert torch.equal(o_pre[0, :Tp - 256], o[:Tp - 256])   # rows of chunks the shorter call shares: the same launches
        steps = []
        for i in range(Tp, T):
            steps.append(yb.gret_decode(q[i][None].contiguous(), k[i][None].contiguous(), v[i][None].contiguous(),
                                        lg[i][None].contiguous(), state, st.scale, group_norm=True, eps=st.eps,
                                        gate=gate[i][None].contiguous())[0])
        got, ref = host(torch.stack(steps)), host(o[Tp:])
        stt = ys.error_stats(got, ref)
        print("bf16 gret stack layer %d, prefill + 8 decode steps vs full forward at the attention output: max_abs %.3e mean_rel %.3e"
              % (n, stt["max_abs"], stt["mean_rel"]), flush=True)
        big = max(1.0, float(np.abs(ref).max()))
        assert stt["max_abs"] <= ys.TOL["bf16"]["max_abs"] * big and stt["mean_rel"] <= ys.TOL["bf16"]["mean_rel"], stt
    # (3) free-running generation
    state = st.new_generation_state(T)
    logits = [host(st.prefill(tok[:T - 8], state))[0]]
    for i in range(T - 8, T):
        logits.append(host(st.decode_step(tok[i], state))[0])
    err = np.abs(np.stack(logits) - full).max()
    print("bf16 gret stack prompt + 8 decode steps vs full forward: %.3e" % err, flush=True)
    assert err <= 0.05 * np.abs(full).max()
