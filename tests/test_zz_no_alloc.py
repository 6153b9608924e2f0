"""yoco_cross_attn_decode_noalloc (the decode step whose split partials live in the library's static device array,
for callers that cannot allocate) against yoco_cross_attn_decode with a caller workspace: same kernels, so the two
outputs must be bit-identical, and both must meet the oracle at the bf16 bounds. Two calls in a row share the static
array, the second with a smaller input: whatever the first call left there must not leak into the second."""
import math

import numpy as np
import pytest
import torch

import oracle
import yoco_synth as ys

pytestmark = pytest.mark.gpu


def one_call(yoco, seed, B, Hq, Hkv, d, N_cap, lens, dtype=torch.bfloat16):
    name = "bf16" if dtype == torch.bfloat16 else "f32"
    scale = 1.0 / math.sqrt(d)
    rng = np.random.default_rng(seed)
    cache = yoco.KVCache(B, Hkv, d, N_cap, dtype)
    cache.mem.zero_()
    K = ys.normal(rng, (B, N_cap, Hkv, d), 1.0, name)
    V = ys.normal(rng, (B, N_cap, Hkv, d), 1.0, name)
    qn = ys.normal(rng, (B, Hq, d), 1.0, name)
    for b in range(B):
        yoco.global_kv_write(cache, torch.from_numpy(K[b]).cuda().to(dtype), torch.from_numpy(V[b]).cuda().to(dtype), b, 0)
    q = torch.from_numpy(qn).cuda().to(dtype)
    lens_t = torch.tensor(lens, dtype=torch.int64, device="cuda")
    nbytes, splits = yoco.cross_attn_decode_workspace(cache, Hq)
    assert nbytes <= yoco.NOALLOC_SCRATCH_BYTES
    ws = torch.full((nbytes // 4,), float("nan"), dtype=torch.float32, device="cuda")
    want = yoco.cross_attn_decode(cache, q, lens_t, scale, ws)
    got = torch.full_like(q, float("nan"))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    yoco.cross_attn_decode_noalloc(cache, q, lens_t, scale, got)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    print("noalloc decode B %d Hq %d Hkv %d d %d N_cap %d splits %d" % (B, Hq, Hkv, d, N_cap, splits), flush=True)
    assert torch.equal(got.view(torch.int16) if dtype == torch.bfloat16 else got.view(torch.int32),
                       want.view(torch.int16) if dtype == torch.bfloat16 else want.view(torch.int32))
    tol = ys.TOL[name]
    for b in range(B):
        n = lens[b]
        ref = oracle.cross_attn(qn[b:b + 1], K[b, :n], V[b, :n], n - 1, scale)[0]
        st = ys.error_stats(got[b].float().cpu().numpy().astype(np.float64), ref)
        assert st["max_abs"] <= tol["max_abs"] and st["mean_rel"] <= tol["mean_rel"], st


def test_noalloc_decode_twice_in_a_row_second_call_smaller(yoco_lib):
    # first call: one long sequence, many splits (the array fills with the partials of tens of splits x 6 heads)
    one_call(yoco_lib, 1, 1, 6, 2, 128, 20000, [19999])
    # second call: smaller in every respect (fewer splits, fewer heads, shorter rows): stale partials must not matter
    one_call(yoco_lib, 2, 2, 4, 2, 128, 700, [700, 13])
    # a shape on the generic kernels (fp32, d = 64), again smaller than the first
    one_call(yoco_lib, 3, 1, 4, 1, 64, 512, [512], dtype=torch.float32)


def test_noalloc_decode_refuses_a_shape_beyond_the_static_array(yoco_lib):
    cache = yoco_lib.KVCache(64, 8, 256, 100, torch.bfloat16)
    nbytes, _ = yoco_lib.cross_attn_decode_workspace(cache, 64)
    assert nbytes > yoco_lib.NOALLOC_SCRATCH_BYTES
    q = torch.zeros(64, 64, 256, dtype=torch.bfloat16, device="cuda")
    out = torch.full_like(q, 7.0)
    with pytest.raises(yoco_lib.YocoError, match="static scratch"):
        yoco_lib.cross_attn_decode_noalloc(cache, q, torch.full((64,), 100, dtype=torch.int64, device="cuda"), 1.0, out)
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())          # a refused call has no side effect


@pytest.fixture(scope="module")
def yoco_lib():
    import paper_2405_05254_amd as y
    y.lib()
    assert torch.cuda.is_available()
    return y
