"""YOCO decoder-decoder stack for the end-to-end early-exit and generation
checks (section 2, Eq. 1-3, Fig. 2 and 3). Attention runs in libyoco; RMSNorm, the projections,
SwiGLU and the classifier are plain torch ops on the GPU (the non-attention
GEMMs are not part of the library).

Precision: the attention operands (Q, K, V, the global cache, O) have the
kernel dtype; the residual stream and the glue GEMMs run in `glue_dtype`
(fp32 by default, with the weights' stored values), so the only bf16 roundings
on the path are the ones at the attention boundary.
"""
import math

import torch

from . import binding as yb


def _rmsnorm(x, gain, eps):
    xf = x.float()
    y = xf * torch.rsqrt(xf.pow(2).mean(-1, keepdim=True) + eps) * gain.float()
    return y.to(x.dtype)


def _rows(x, fn, chunk=16384):
    """Apply a row-wise function in row chunks (bounds the FFN intermediates at long T)."""
    if x.shape[0] <= chunk:
        return fn(x)
    return torch.cat([fn(x[i:i + chunk]) for i in range(0, x.shape[0], chunk)])


def _swiglu(x, L):
    return (torch.nn.functional.silu(x @ L["W_G"]) * (x @ L["W_1"])) @ L["W_2"]


class YocoStack:
    """weights: the dict produced by the synthetic generator (numpy arrays);
    dtype: torch.float32 or torch.bfloat16."""

    def __init__(self, weights, dtype, device="cuda", glue_dtype=torch.float32, cache_dtype=None, fused_kv_norm=False):
        self.dtype, self.device, self.glue = dtype, device, glue_dtype
        self.cache_dtype = dtype if cache_dtype is None else cache_dtype   # torch.int8: the global cache holds 8-bit codes
        self.fused_kv_norm = fused_kv_norm   # Eq. 2 with the norm's 1/rms folded into the cache write (yoco_global_kv_write_scaled)
        self.capture = None          # dict layer-name -> (q, k, v, o) (gated retention: + log-decays, gate) when set by a test

        def dev(a):
            return torch.as_tensor(a).to(device=device, dtype=glue_dtype)

        def layer(L):
            return {k: dev(v) for k, v in L.items()}

        w = weights
        self.Hq, self.Hkv_self, self.Hkv, self.d = w["Hq"], w["Hkv_self"], w["Hkv"], w["d"]
        self.window, self.eps = w["window"], w["eps"]
        self.self_kind, self.tau = w.get("self_kind", "swa"), w.get("tau", 16.0)   # "swa" (Eq. 8) or "gret" (Eq. 7)
        self.scale = 1.0 / math.sqrt(self.d)
        self.embed = dev(w["embed"])
        self.self_layers = [layer(L) for L in w["self"]]
        self.kv = layer(w["kv"])
        if fused_kv_norm:             # gain-scaled weights diag(g) W_K, diag(g) W_V, formed once
            self.kv["gW_K"] = (self.kv["ln"].float()[:, None] * self.kv["W_K"].float()).to(glue_dtype)
            self.kv["gW_V"] = (self.kv["ln"].float()[:, None] * self.kv["W_V"].float()).to(glue_dtype)
        self.cross_layers = [layer(L) for L in w["cross"]]
        self.final_ln, self.W_out = dev(w["final_ln"]), dev(w["W_out"])

    # -- self-decoder: Eq. 1 with sliding-window attention (Eq. 8)
    def _log_decay(self, xn, L):
        """ln(gamma) of Eq. 4: logsigmoid(x W_gamma) / tau, float32 [rows, H]."""
        return (torch.nn.functional.logsigmoid(xn.float() @ L["W_gamma"].float()) / self.tau).contiguous()

    def self_decoder(self, tokens, rings=None):
        """rings: optional per-layer generation caches that receive what a later decode step needs: rolling
        caches (the last `window` K/V rows) for sliding-window attention, fp32 states for gated retention."""
        X = self.embed[tokens]
        T = X.shape[0]
        for n, L in enumerate(self.self_layers):
            xn = _rmsnorm(X, L["ln1"], self.eps)
            q = (xn @ L["W_Q"]).to(self.dtype).view(1, T, self.Hq, self.d)
            k = (xn @ L["W_K"]).to(self.dtype).view(1, T, self.Hkv_self, self.d)
            v = (xn @ L["W_V"]).to(self.dtype).view(1, T, self.Hkv_self, self.d)
            if self.self_kind == "gret":
                lg = self._log_decay(xn, L).view(1, T, self.Hq)
                code = yb.F32 if self.dtype == torch.float32 else yb.BF16
                nbytes = yb.gret_prefill_workspace(1, T, self.Hq, self.d, self.d, 256, code)
                ws = torch.empty(nbytes, dtype=torch.uint8, device=self.device) if nbytes else None
                gate = (xn @ L["W_gate"]).to(self.dtype).view(1, T, self.Hq, self.d)
                o = yb.gret_prefill(q, k, v, lg, self.scale, chunk=256, group_norm=True, eps=self.eps,
                                    state_out=None if rings is None else rings[n], workspace=ws, gate=gate)
                a = o.view(T, self.Hq * self.d).to(self.glue)
                if self.capture is not None and ("self%d" % n) in self.capture:
                    self.capture["self%d" % n] = (q[0], k[0], v[0], o[0], lg[0], gate[0])
                del ws, lg, gate
            else:
                o = yb.swa_prefill(q, k, v, self.window, self.scale)
                if rings is not None:
                    yb.swa_cache_write(rings[n], k[0], v[0], 0, 0)
                a = o.view(T, self.Hq * self.d).to(self.glue)
            if self.capture is not None and self.self_kind != "gret" and ("self%d" % n) in self.capture:
                self.capture["self%d" % n] = (q[0], k[0], v[0], o[0])
            Y = a @ L["W_O"] + X
            del q, k, v, o, xn, a
            X = _rows(Y, lambda y: _swiglu(_rmsnorm(y, L["ln2"], self.eps), L) + y)
        return X

    # -- Eq. 2: the global cache, written once
    def write_cache(self, X, cache=None, pos0=0):
        T = X.shape[0]
        if cache is None:
            cache = yb.KVCache(1, self.Hkv, self.d, T, self.cache_dtype, self.device)
        if self.fused_kv_norm:
            # RMSNorm(x) W = (1 / rms(x)) (x (diag(g) W)): no normalised copy of X, the factor rides on the write
            rs = torch.rsqrt(torch.linalg.vector_norm(X, dim=-1, dtype=torch.float32).pow(2) / X.shape[-1] + self.eps).contiguous()
            k = (X @ self.kv["gW_K"]).view(T, self.Hkv, self.d)
            v = (X @ self.kv["gW_V"]).view(T, self.Hkv, self.d)
            yb.global_kv_write_scaled(cache, k, v, rs, 0, pos0)
            return cache
        xn = _rmsnorm(X, self.kv["ln"], self.eps)
        k = (xn @ self.kv["W_K"]).to(self.dtype).view(T, self.Hkv, self.d)
        v = (xn @ self.kv["W_V"]).to(self.dtype).view(T, self.Hkv, self.d)
        yb.global_kv_write(cache, k, v, 0, pos0)
        return cache

    # -- cross-decoder: Eq. 3
    def _cross_layer(self, X, L, attn):
        Tq = X.shape[0]
        q = (_rmsnorm(X, L["ln1"], self.eps) @ L["W_Q"]).to(self.dtype).view(Tq, self.Hq, self.d)
        a = attn(q).view(Tq, self.Hq * self.d).to(self.glue)
        Y = a @ L["W_O"] + X
        del q, a
        return _rows(Y, lambda y: _swiglu(_rmsnorm(y, L["ln2"], self.eps), L) + y)

    def cross_decoder_rows(self, X, cache, q_pos0):
        ws = None
        if X.shape[0] <= 8:          # few rows: let the call split over the cache
            nbytes, _ = yb.cross_attn_decode_workspace(cache, self.Hq)
            ws = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        for n, L in enumerate(self.cross_layers):
            def attn(q, n=n):
                o = yb.cross_attn_prefill(cache, q, 0, q_pos0, self.scale, workspace=ws)
                if self.capture is not None and ("cross%d" % n) in self.capture:
                    self.capture["cross%d" % n] = (q, o)
                return o
            X = self._cross_layer(X, L, attn)
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

    # -- token-by-token generation (Fig. 3 "Generation"): rolling caches in the self-decoder
    def new_generation_state(self, max_len):
        """Caches of one sequence: per self-decoder layer a ring of `window` rows (sliding-window attention) or an
        fp32 state (gated retention), and the global cache."""
        if self.self_kind == "gret":
            rings = [torch.zeros(1, self.Hq, self.d, self.d, dtype=torch.float32, device=self.device) for _ in self.self_layers]
        else:
            rings = [yb.KVCache(1, self.Hkv_self, self.d, self.window, self.dtype, self.device) for _ in self.self_layers]
        cache = yb.KVCache(1, self.Hkv, self.d, max_len, self.cache_dtype, self.device)
        ws = []
        for c in ((cache, cache) if self.self_kind == "gret" else (rings[0], cache)):
            nbytes, _ = yb.cross_attn_decode_workspace(c, self.Hq)
            ws.append(torch.empty(nbytes, dtype=torch.uint8, device=self.device))
        return dict(rings=rings, cache=cache, ws_ring=ws[0], ws_cache=ws[1], length=0)

    def prefill(self, tokens, state):
        """Early-exit prefill of a prompt (state must be fresh); returns the logits of its last position."""
        assert state["length"] == 0
        X = self.self_decoder(tokens, rings=state["rings"])
        T = X.shape[0]
        self.write_cache(X, state["cache"], 0)
        state["length"] = T
        lens = torch.tensor([T], dtype=torch.int64, device=self.device)
        x = X[T - 1:T].contiguous()
        for L in self.cross_layers:
            x = self._cross_layer(x, L, lambda q: yb.cross_attn_decode(state["cache"], q, lens, self.scale, state["ws_cache"]))
        return self.logits(x)

    def decode_step(self, token, state):
        """One new token through both decoders; returns its logits [1,vocab]."""
        p = state["length"]
        pos = torch.tensor([p], dtype=torch.int64, device=self.device)
        lens = pos + 1
        x = self.embed[torch.as_tensor(token, device=self.device).view(1)]
        for L, ring in zip(self.self_layers, state["rings"]):
            xn = _rmsnorm(x, L["ln1"], self.eps)
            q = (xn @ L["W_Q"]).to(self.dtype).view(1, self.Hq, self.d)
            k = (xn @ L["W_K"]).to(self.dtype).view(1, self.Hkv_self, self.d)
            v = (xn @ L["W_V"]).to(self.dtype).view(1, self.Hkv_self, self.d)
            if self.self_kind == "gret":
                gate = (xn @ L["W_gate"]).to(self.dtype).view(1, self.Hq, self.d)
                o = yb.gret_decode(q, k, v, self._log_decay(xn, L).view(1, self.Hq), ring, self.scale, group_norm=True,
                                   eps=self.eps, gate=gate)
                a = o.view(1, self.Hq * self.d).to(self.glue)
            else:
                o = yb.swa_decode(ring, q, lens, self.scale, state["ws_ring"], k_new=k, v_new=v)   # appends the row itself
                a = o.view(1, self.Hq * self.d).to(self.glue)
            y = a @ L["W_O"] + x
            x = _swiglu(_rmsnorm(y, L["ln2"], self.eps), L) + y
        xn = _rmsnorm(x, self.kv["ln"], self.eps)
        k = (xn @ self.kv["W_K"]).to(self.dtype).view(1, self.Hkv, self.d)
        v = (xn @ self.kv["W_V"]).to(self.dtype).view(1, self.Hkv, self.d)
        yb.kv_cache_append(state["cache"], k, v, pos, False)
        for L in self.cross_layers:
            x = self._cross_layer(x, L, lambda q: yb.cross_attn_decode(state["cache"], q, lens, self.scale, state["ws_cache"]))
        state["length"] = p + 1
        return self.logits(x)
