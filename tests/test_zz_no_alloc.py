"""The allocation-free decode entry point (flashcache_decode_attention_static) through the C ABI.

It runs the kernels of flashcache_decode_attention with the partial results in the library's own
fixed device array, so its output must equal that entry point's bit for bit; checked on two calls
in a row, the second with a smaller input (the array then still holds the first call's records),
and against the oracle at the decode tolerance.  Oversized shapes are refused before any launch.
"""
import numpy as np
import pytest

import kvsynth
from oracle import flashcache_ref as ref

import parity_util as pu

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _case(fc, rng, dtype, B, L, H, Hq, d, N):
    budgets = rng.integers(0, N // 2 + 1, (B, L)).astype(np.int64)
    budgets[:, 0] = N // 3                                         # every sequence: same packed row count
    budgets[:, 1:] = budgets[0, 1:]
    offs = np.stack([ref.layer_offsets(budgets[b], H) for b in range(B)])
    rows = int(offs[0, -1])

    def make(shape, sigma=1.0):
        x = (sigma * rng.standard_normal(shape)).astype(np.float32)
        return kvsynth.f32_to_bf16_bits(x) if dtype == "bf16" else x
    Kr, Vr, Q = make((B, rows, d)), make((B, rows, d), 2.0), make((B, L, Hq, d))
    return budgets, offs, rows, Kr, Vr, Q


@pytest.mark.parametrize("dtype,d,Hq,H", [("bf16", 128, 28, 4), ("f32", 64, 4, 2)])
def test_static_scratch_decode_matches_workspace_variant_twice(dtype, d, Hq, H):
    import paper_2511_16786_amd as fc
    rng = np.random.default_rng(99 + d)
    scale = float(1.0 / np.sqrt(d))
    assert fc.decode_static_scratch_bytes() == 16 << 20
    for B, L, N in ((2, 6, 5000), (1, 2, 700)):                    # the second call is the smaller one
        budgets, offs, rows, Kr, Vr, Q = _case(fc, rng, dtype, B, L, H, Hq, d, N)
        Qt, Kt, Vt = pu.to_torch(Q, dtype), pu.to_torch(Kr, dtype), pu.to_torch(Vr, dtype)
        b_t = torch.from_numpy(budgets.astype(np.int32)).cuda()
        o_t = torch.from_numpy(offs).cuda()
        want = fc.decode_attention(Qt, Kt, Vt, H, b_t, o_t, rows, scale)
        got = torch.full((B, L, Hq, d), float("nan"), dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        fc.decode_attention_static(Qt, Kt, Vt, H, b_t, o_t, rows, scale, got)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before              # nothing came from torch's allocator
        assert torch.equal(got, want), f"static-scratch result differs from the workspace variant (B={B}, L={L})"
        vmax = float(np.abs(ref.widen(Vr, dtype)).max())
        for b in range(B):
            oracle = ref.decode_attention(Q[b], Kr[b], Vr[b], dtype, budgets[b], H, scale)
            assert np.abs(got[b].cpu().numpy() - oracle).max() <= 5e-5 * vmax


def test_static_scratch_refuses_shapes_beyond_its_size():
    import paper_2511_16786_amd as fc
    from paper_2511_16786_amd import binding as b
    # 8 x 64 x 8 units of 16 query heads each: the partial records need more than the 16 MiB array
    B, L, H, Hq, d = 8, 64, 8, 128, 128
    need = int(b._lib.flashcache_decode_workspace_bytes(B, L, H, Hq, d))
    assert need > fc.decode_static_scratch_bytes()
    st = b._lib.flashcache_decode_attention_static(256, 256, 256, B, L, H, Hq, d, b.FC_BF16, 256, 256, 0, 1.0,
                                                   256, None)
    assert st == b.FC_EWORKSPACE
