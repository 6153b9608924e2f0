"""The generation calls are plain kernel launches on the caller's stream (no
allocation, no memset, no synchronisation), so a decode step can be captured
into a HIP graph. One step of a 3 + 3-layer stack's attention (rolling-window
append + decode, gated-retention decode, global-cache append + split-KV decode,
the same over an 8-bit global cache) is captured once and replayed several times with eager work and
synchronisations in between; every replay must reproduce the eager result bit
for bit."""
import math

import numpy as np
import pytest
import torch

import yoco_synth as ys

pytestmark = pytest.mark.gpu


def test_decode_step_replays_from_a_hip_graph():
    import paper_2405_05254_amd as yoco
    yoco.lib()
    B, H, Hkv, d, C, N, layers = 4, 8, 4, 128, 256, 2048, 3
    scale = 1.0 / math.sqrt(d)
    dev = "cuda"
    bf = torch.bfloat16
    rings = [yoco.KVCache(B, H, d, C, bf) for _ in range(layers)]
    cache = yoco.KVCache(B, Hkv, d, N, bf)
    for i, kv in enumerate(rings + [cache]):
        for pl in kv.planes():
            pl.copy_(ys.device_normal(pl.shape, 40 + i, 1.0, bf, dev))
    cache8 = yoco.KVCache(B, Hkv, d, N, torch.int8)     # the 8-bit variant of the global cache, filled by the write call
    for b in range(B):
        yoco.global_kv_write(cache8, ys.device_normal((N, Hkv, d), 50 + b, 1.0, bf, dev), ys.device_normal((N, Hkv, d), 55 + b, 1.0, bf, dev), b, 0)
    states0 = [ys.device_normal((B, H, d, d), 60 + i, 1.0, torch.float32, dev) for i in range(layers)]
    q = [ys.device_normal((B, H, d), 70 + i, 1.0, bf, dev) for i in range(3 * layers)]
    knew = [ys.device_normal((B, H, d), 90 + i, 1.0, bf, dev) for i in range(layers)]
    khat = ys.device_normal((B, Hkv, d), 99, 1.0, bf, dev)
    lg = -torch.rand(B, H, device=dev) * 0.1
    pos = torch.tensor([1000, 1500, 300, 2047], dtype=torch.int64, device=dev)
    lens = pos + 1
    ws_r = torch.empty(yoco.cross_attn_decode_workspace(rings[0], H)[0], dtype=torch.uint8, device=dev)
    ws_c = torch.empty(yoco.cross_attn_decode_workspace(cache, H)[0], dtype=torch.uint8, device=dev)
    states = [s.clone() for s in states0]
    ws_8 = torch.empty(yoco.cross_attn_decode_workspace(cache8, H)[0], dtype=torch.uint8, device=dev)
    outs = [torch.empty(B, H, d, dtype=bf, device=dev) for _ in range(3 * layers + 1)]

    def step():
        for i in range(layers):
            yoco.kv_cache_append(rings[i], knew[i], knew[i], pos, True)
            yoco.swa_decode(rings[i], q[i], lens, scale, ws_r, out=outs[i])
            yoco.gret_decode(q[layers + i], knew[i], knew[i], lg, states[i], scale, out=outs[layers + i])
        yoco.kv_cache_append(cache, khat, khat, pos, False)
        for i in range(layers):
            yoco.cross_attn_decode(cache, q[2 * layers + i], lens, scale, ws_c, out=outs[2 * layers + i])
        yoco.kv_cache_append(cache8, khat, khat, pos, False)
        yoco.cross_attn_decode(cache8, q[0], lens, scale, ws_8, out=outs[3 * layers])

    def reset():
        for s, s0 in zip(states, states0):
            s.copy_(s0)                           # the retention state advances with every step: start each run alike

    reset()
    step()
    torch.cuda.synchronize()
    want = [o.clone() for o in outs]
    want_states = [s.clone() for s in states]

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    reset()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for rep in range(4):
        reset()
        for o in outs:
            o.zero_()
        junk = torch.randn(1 << 20, device=dev).sum()        # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert math.isfinite(float(junk))
        for i, (o, w) in enumerate(zip(outs, want)):
            assert torch.equal(o, w), "output %d differs on replay %d" % (i, rep)
        for s, w in zip(states, want_states):
            assert torch.equal(s, w), "a retention state differs on replay %d" % rep
    assert np.isfinite(want[0].float().cpu().numpy()).all()
