"""YOCO decoder-decoder stack for the end-to-end early-exit check (section 2,
Eq. 1-3, Fig. 2 and 3). Attention runs in libyoco; RMSNorm, the projections,
SwiGLU and the classifier are plain torch ops on the GPU (the non-attention
GEMMs are not part of the library).
"""
import math

import torch

from . import binding as yb


def _rmsnorm(x, gain, eps):
    xf = x.float()
    y = xf * torch.rsqrt(xf.pow(2).mean(-1, keepdim=True) + eps) * gain.float()
    return y.to(x.dtype)


def _swiglu(x, L):
    return (torch.nn.functional.silu(x @ L["W_G"]) * (x @ L["W_1"])) @ L["W_2"]


class YocoStack:
    """weights: the dict produced by the synthetic generator (numpy arrays);
    dtype: torch.float32 or torch.bfloat16."""

    def __init__(self, weights, dtype, device="cuda"):
        self.dtype, self.device = dtype, device

        def dev(a):
            return torch.as_tensor(a).to(device=device, dtype=dtype)

        def layer(L):
            return {k: dev(v) for k, v in L.items()}

        w = weights
        self.Hq, self.Hkv_self, self.Hkv, self.d = w["Hq"], w["Hkv_self"], w["Hkv"], w["d"]
        self.window, self.eps = w["window"], w["eps"]
        self.scale = 1.0 / math.sqrt(self.d)
        self.embed = dev(w["embed"])
        self.self_layers = [layer(L) for L in w["self"]]
        self.kv = layer(w["kv"])
        self.cross_layers = [layer(L) for L in w["cross"]]
        self.final_ln, self.W_out = dev(w["final_ln"]), dev(w["W_out"])

    # -- self-decoder: Eq. 1 with sliding-window attention (Eq. 8)
    def self_decoder(self, tokens):
        X = self.embed[tokens]
        T = X.shape[0]
        for L in self.self_layers:
            xn = _rmsnorm(X, L["ln1"], self.eps)
            q = (xn @ L["W_Q"]).view(1, T, self.Hq, self.d)
            k = (xn @ L["W_K"]).view(1, T, self.Hkv_self, self.d)
            v = (xn @ L["W_V"]).view(1, T, self.Hkv_self, self.d)
            a = yb.swa_prefill(q, k, v, self.window, self.scale).view(T, self.Hq * self.d)
            Y = a @ L["W_O"] + X
            X = _swiglu(_rmsnorm(Y, L["ln2"], self.eps), L) + Y
        return X

    # -- Eq. 2: the global cache, written once
    def write_cache(self, X, cache=None, pos0=0):
        T = X.shape[0]
        xn = _rmsnorm(X, self.kv["ln"], self.eps)
        k = (xn @ self.kv["W_K"]).view(T, self.Hkv, self.d)
        v = (xn @ self.kv["W_V"]).view(T, self.Hkv, self.d)
        if cache is None:
            cache = yb.KVCache(1, self.Hkv, self.d, T, self.dtype, self.device)
        yb.global_kv_write(cache, k, v, 0, pos0)
        return cache

    # -- cross-decoder: Eq. 3
    def _cross_layer(self, X, L, attn):
        Tq = X.shape[0]
        q = (_rmsnorm(X, L["ln1"], self.eps) @ L["W_Q"]).view(Tq, self.Hq, self.d)
        a = attn(q).view(Tq, self.Hq * self.d)
        Y = a @ L["W_O"] + X
        return _swiglu(_rmsnorm(Y, L["ln2"], self.eps), L) + Y

    def cross_decoder_rows(self, X, cache, q_pos0):
        for L in self.cross_layers:
            X = self._cross_layer(X, L, lambda q: yb.cross_attn_prefill(cache, q, 0, q_pos0, self.scale))
        return X

    def cross_decoder_decode(self, x_last, cache, length):
        """One token through the cross-decoder with the split-KV decode kernel."""
        nbytes, _ = yb.cross_attn_decode_workspace(cache, self.Hq)
        ws = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        lens = torch.tensor([length], dtype=torch.int64, device=self.device)
        X = x_last
        for L in self.cross_layers:
            X = self._cross_layer(X, L, lambda q: yb.cross_attn_decode(cache, q, lens, self.scale, ws))
        return X

    def logits(self, X):
        return _rmsnorm(X, self.final_ln, self.eps) @ self.W_out

    def forward_full(self, tokens, rows=None):
        """Every row through both decoders; logits of `rows` (default: all)."""
        X = self.self_decoder(tokens)
        cache = self.write_cache(X)
        X = self.cross_decoder_rows(X, cache, 0)
        return self.logits(X if rows is None else X[rows])

    def forward_early_exit(self, tokens, decode_kernel=True):
        """Prefill that leaves after the self-decoder and the cache write; only
        the last position enters the cross-decoder (Fig. 3)."""
        X = self.self_decoder(tokens)
        T = X.shape[0]
        cache = self.write_cache(X)
        x_last = X[T - 1:T].contiguous()
        if decode_kernel:
            x_last = self.cross_decoder_decode(x_last, cache, T)
        else:
            x_last = self.cross_decoder_rows(x_last, cache, T - 1)
        return self.logits(x_last), cache
