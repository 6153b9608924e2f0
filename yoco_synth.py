"""Seeded synthetic inputs for the YOCO attention hot path, and error metrics.

This module holds none of the method's arithmetic: it only draws random
numbers, rounds them to the storage dtype, and names the five workload
configurations. Both the tests of the HIP library and the fp64 oracle consume
what it produces, so the two sides see identical bits.

Shapes follow the paper's own profiling setup (section 4.4 with the 3B
configuration of section 4.1 / appendix C: 24 query heads, 8 KV heads, head
dimension 128, 26 layers = 13 + 13; window 1024 from section 4.2; the 1.4B row
of the scaling table in appendix D for the end-to-end stack). The paper's
measurements use its own prompts of 32K-1M tokens, not a public dataset; normal
random tensors of those shapes stand in for them.
"""
import numpy as np

CONFIGS = {
    # Tiny fp32 case the oracle finishes in seconds.
    "tiny_fp32": dict(dtype="f32", T=512, d=64, swa=dict(Hq=4, Hkv=4, window=128, std=1.0),
                      cross=dict(Hq=4, Hkv=1, std=1.0),
                      stack=dict(d_model=256, Hq=4, Hkv_self=4, Hkv=1, d=64, n_self=2, n_cross=2,
                                 window=128, ffn=704, vocab=1000, eps=1e-6), seed=0),
    # SWA prefill, the configuration the headline metric is quoted on.
    "swa_prefill_32k": dict(dtype="bf16", B=1, T=32768, Hq=24, Hkv=24, d=128, window=1024, std=0.5, seed=0),
    # Batched decode over 16 caches of 32K tokens, 13 cross-decoder layers.
    "decode_b16_32k": dict(dtype="bf16", B=16, N=32768, Hq=24, Hkv=8, d=128, layers=13, std=1.0, seed=0),
    # Long-context decode over one cache of 512K tokens, 13 cross-decoder layers.
    "decode_b1_512k": dict(dtype="bf16", B=1, N=524288, Hq=24, Hkv=8, d=128, layers=13, std=1.0, seed=0),
    # End-to-end early-exit prefill of a random-init stack.
    "e2e_early_exit_128k": dict(dtype="bf16", B=1, T=131072,
                                stack=dict(d_model=2048, Hq=16, Hkv_self=16, Hkv=16, d=128, n_self=12,
                                           n_cross=12, window=1024, ffn=5632, vocab=32000, eps=1e-6), seed=0),
}


# ---------------------------------------------------------------- bf16 storage
def f32_to_bf16_bits(x):
    """float32 array -> uint16 bf16 bit patterns, round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + r) >> 16).astype(np.uint16)


def bf16_bits_to_f32(b):
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def round_to(x, dtype):
    """Round a float32 array to the storage dtype and return it as float32."""
    if dtype == "bf16":
        return bf16_bits_to_f32(f32_to_bf16_bits(x))
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    raise ValueError(dtype)


def normal(rng, shape, std, dtype):
    """std * N(0,1) drawn in float32, rounded once to the storage dtype."""
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    return round_to(x, dtype)


def qkv(seed, T, Hq, Hkv, d, std, dtype):
    rng = np.random.default_rng(seed)
    return (normal(rng, (T, Hq, d), std, dtype), normal(rng, (T, Hkv, d), std, dtype),
            normal(rng, (T, Hkv, d), std, dtype))


def gret_inputs(seed, B, T, H, dk, dv, std, dtype, mean_log_decay=0.04):
    """Inputs of gated retention: q, k [B,T,H,dk], v [B,T,H,dv] as for attention, and the log-decays
    ln(gamma) [B,T,H] in float32, drawn as minus an exponential variate (gamma in (0, 1), mostly 0.9-1:
    the range a sigmoid raised to 1/16 produces)."""
    rng = np.random.default_rng(seed)
    q = normal(rng, (B, T, H, dk), std, dtype)
    k = normal(rng, (B, T, H, dk), std, dtype)
    v = normal(rng, (B, T, H, dv), std, dtype)
    lg = (-rng.exponential(mean_log_decay, size=(B, T, H))).astype(np.float32)
    return q, k, v, lg


def stack_weights(seed, s, dtype):
    """Random-init YOCO stack: matrices ~ N(0, 0.02), RMSNorm gains 1, no bias."""
    rng = np.random.default_rng(seed)
    dm, Hq, d, ffn = s["d_model"], s["Hq"], s["d"], s["ffn"]

    def mat(*shape):
        return normal(rng, shape, 0.02, dtype)

    def ones():
        return np.ones(dm, dtype=np.float32)

    def ffn_w():
        return dict(ln2=ones(), W_G=mat(dm, ffn), W_1=mat(dm, ffn), W_2=mat(ffn, dm))

    w = dict(Hq=Hq, Hkv_self=s["Hkv_self"], Hkv=s["Hkv"], d=d, window=s["window"], eps=s["eps"])
    w["embed"] = mat(s["vocab"], dm)
    w["self"] = [dict(ln1=ones(), W_Q=mat(dm, Hq * d), W_K=mat(dm, s["Hkv_self"] * d),
                      W_V=mat(dm, s["Hkv_self"] * d), W_O=mat(Hq * d, dm), **ffn_w())
                 for _ in range(s["n_self"])]
    w["kv"] = dict(ln=ones(), W_K=mat(dm, s["Hkv"] * d), W_V=mat(dm, s["Hkv"] * d))
    w["cross"] = [dict(ln1=ones(), W_Q=mat(dm, Hq * d), W_O=mat(Hq * d, dm), **ffn_w())
                  for _ in range(s["n_cross"])]
    w["final_ln"] = ones()
    w["W_out"] = mat(dm, s["vocab"])
    if s.get("self_kind", "swa") == "gret":           # gated-retention self-decoder: decay and gate projections
        w["self_kind"], w["tau"] = "gret", s.get("tau", 16.0)
        for L in w["self"]:                           # drawn last, so the other matrices match the SWA variant's
            L["W_gamma"] = normal(rng, (dm, Hq), 1.0, dtype)
            L["W_gate"] = mat(dm, Hq * d)
    return w


def stack_weights_device(seed, s, torch_dtype, device):
    """The same random-init stack drawn on the device (the 1.4B-parameter
    end-to-end configuration): N(0, 0.02) rounded to `torch_dtype`, gains 1."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    dm, Hq, d, ffn = s["d_model"], s["Hq"], s["d"], s["ffn"]

    def mat(*shape):
        x = torch.empty(shape, dtype=torch.float32, device=device)
        x.normal_(0.0, 0.02, generator=g)
        return x.to(torch_dtype)

    def ones():
        return torch.ones(dm, dtype=torch.float32, device=device)

    def ffn_w():
        return dict(ln2=ones(), W_G=mat(dm, ffn), W_1=mat(dm, ffn), W_2=mat(ffn, dm))

    w = dict(Hq=Hq, Hkv_self=s["Hkv_self"], Hkv=s["Hkv"], d=d, window=s["window"], eps=s["eps"])
    w["embed"] = mat(s["vocab"], dm)
    w["self"] = [dict(ln1=ones(), W_Q=mat(dm, Hq * d), W_K=mat(dm, s["Hkv_self"] * d),
                      W_V=mat(dm, s["Hkv_self"] * d), W_O=mat(Hq * d, dm), **ffn_w())
                 for _ in range(s["n_self"])]
    w["kv"] = dict(ln=ones(), W_K=mat(dm, s["Hkv"] * d), W_V=mat(dm, s["Hkv"] * d))
    w["cross"] = [dict(ln1=ones(), W_Q=mat(dm, Hq * d), W_O=mat(Hq * d, dm), **ffn_w())
                  for _ in range(s["n_cross"])]
    w["final_ln"] = ones()
    w["W_out"] = mat(dm, s["vocab"])
    return w


def tokens(seed, T, vocab):
    return np.random.default_rng(seed + 7919).integers(0, vocab, size=T, dtype=np.int64)


def device_normal(shape, seed, std, torch_dtype, device):
    """Large tensors (the 2 GB caches) are drawn on the device with a seeded
    torch generator; the host reads back the same bits for the oracle."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    x = torch.empty(shape, dtype=torch.float32, device=device)
    x.normal_(0.0, std, generator=g)
    return x.to(torch_dtype)


# ---------------------------------------------------------------- error metrics
def error_stats(got, ref):
    """max |got-ref| and sum|got-ref| / sum|ref| (ratio of sums: element-wise
    ratios blow up where the reference is near zero)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    diff = np.abs(got - ref)
    denom = np.abs(ref).sum()
    return dict(max_abs=float(diff.max()) if diff.size else 0.0,
                mean_rel=float(diff.sum() / denom) if denom > 0 else 0.0,
                argmax=int(diff.argmax()) if diff.size else -1)


TOL = {"bf16": dict(max_abs=2e-2, mean_rel=2e-3), "f32": dict(max_abs=1e-4, mean_rel=1e-4)}
