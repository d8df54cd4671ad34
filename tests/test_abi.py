"""The C-ABI library loads, exports every declared symbol, and validates on the host.

No GPU is touched: the calls below either are host helpers or fail validation before any
HIP call is made.
"""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2511_16786_amd", "libflashcache.so")

pytestmark = pytest.mark.skipif(not os.path.exists(LIB), reason="libflashcache.so not built")


def _declared_symbols():
    with open(os.path.join(ROOT, "include", "flashcache.h")) as f:
        text = f.read()
    return sorted(set(re.findall(r"\b(flashcache_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    lib = ctypes.CDLL(LIB)
    names = _declared_symbols()
    assert len(names) >= 10
    for name in names:
        assert hasattr(lib, name), name


def test_binding_lists_the_same_symbols():
    from paper_2511_16786_amd import binding
    assert sorted(binding.EXPORTED_SYMBOLS) == _declared_symbols()


def test_host_helpers_match_documented_rounding():
    import paper_2511_16786_amd as fc
    assert [fc.cutoff_r(n, g) for n, g in [(512, .1), (4096, .1), (8192, .1), (32768, .05), (16384, .1)]] \
        == [52, 410, 820, 1639, 1639]
    assert fc.cutoff_r(10, 0.0) == 1 and fc.cutoff_r(10, 1.0) == 10 and fc.cutoff_r(10, 5.0) == 10
    assert fc.cutoff_r(0, 0.1) == 0 and fc.cutoff_r(10, float("nan")) == 1
    assert [fc.total_budget(l, n, r) for l, n, r in
            [(1, 512, .2), (4, 4096, .2), (28, 8192, .2), (28, 32768, .2), (28, 16384, .1)]] \
        == [102, 3276, 45875, 183500, 45875]
    assert fc.total_budget(4, 100, 0.0) == 4 and fc.total_budget(4, 100, 2.0) == 400


def _desc(fc, B=1, L=2, H=2, N=64, d=64, dtype=0):
    return fc.FcKvDesc(B, L, H, N, d, dtype, L * H * N * d, H * N * d, N * d, d)


def test_validation_errors_before_any_launch():
    import paper_2511_16786_amd as fc
    from paper_2511_16786_amd import binding as b
    lib = b._lib
    d = _desc(fc)
    ref = ctypes.byref
    # r outside [1, N]
    assert lib.flashcache_score(16, 16, ref(d), 0, 1, 16, 16, 256, 1 << 30, None) == b.FC_EINVAL
    assert lib.flashcache_score(16, 16, ref(d), 65, 1, 16, 16, 256, 1 << 30, None) == b.FC_EINVAL
    # null pointers
    assert lib.flashcache_score(None, 16, ref(d), 7, 1, 16, 16, 256, 1 << 30, None) == b.FC_EINVAL
    # workspace missing / too small / misaligned
    assert lib.flashcache_score(16, 16, ref(d), 7, 1, 16, 16, None, 0, None) == b.FC_EWORKSPACE
    assert lib.flashcache_score(16, 16, ref(d), 7, 1, 16, 16, 256, 16, None) == b.FC_EWORKSPACE
    assert lib.flashcache_score(16, 16, ref(d), 7, 1, 16, 16, 264, 1 << 30, None) == b.FC_EWORKSPACE
    # head dim whose rows are not multiples of 16 bytes; bad dtype
    bad = _desc(fc, d=6)
    assert lib.flashcache_score(16, 16, ref(bad), 7, 1, 16, 16, 256, 1 << 30, None) == b.FC_EINVAL
    bad = _desc(fc, dtype=7)
    assert lib.flashcache_prepare(ref(bad), 7, 1, 256, 1 << 30, None) == b.FC_EINVAL
    # dense realisation: any head dim up to 256 whose rows are multiples of 16 bytes
    wide = _desc(fc, d=320)
    assert lib.flashcache_prepare(ref(wide), 7, b.FC_PATH_DENSE, 256, 1 << 30, None) == b.FC_EUNSUPPORTED
    assert fc.workspace_bytes(wide, 7, b.FC_PATH_DENSE) == 0
    assert fc.workspace_bytes(_desc(fc, d=40), 7, b.FC_PATH_DENSE) == fc.workspace_bytes(_desc(fc, d=64), 7, b.FC_PATH_DENSE)
    # the fast transform needs a token count that is a multiple of 256 whose tables fit LDS
    # (multiples of 1024 up to 132 * 1024, multiples of 512 or 256 up to 64 * 1024, these with d % 16 == 0) ...
    np2 = _desc(fc, N=1000, d=128, dtype=1)
    assert fc.resolve_path(np2, 100, b.FC_PATH_FFT) == 0
    assert fc.resolve_path(np2, 100, b.FC_PATH_AUTO) == b.FC_PATH_DENSE
    def fast(N, d_=128):
        return fc.resolve_path(_desc(fc, L=1, H=1, N=N, d=d_, dtype=1), 100, b.FC_PATH_FFT) == b.FC_PATH_FFT
    assert fast(128 * 1024) and fast(132 * 1024) and not fast(133 * 1024) and not fast(256 * 1024)
    assert fast(64000) and fast(32000) and fast(65536 - 256) and fast(65536 - 512)
    assert not fast(32000 + 128) and not fast(64000, d_=24) and fast(64512, d_=24)
    # ... and takes any cut-off 1 <= r <= N (several passes above 2048 modes, complement mode above N/2),
    # with a workspace that grows by the fp32 buffer of the passes only when there are several
    m3 = _desc(fc, N=3072, d=128, dtype=1)
    for r in (1, 1024, 1536, 1537, 2048, 3071, 3072):
        assert fc.resolve_path(m3, r, b.FC_PATH_AUTO) == b.FC_PATH_FFT, r
    m16 = _desc(fc, N=16384, d=128, dtype=1)
    one_pass = fc.workspace_bytes(m16, 2048, b.FC_PATH_FFT)
    assert fc.workspace_bytes(m16, 16384 - 2047, b.FC_PATH_FFT) == one_pass        # complement, one pass
    # cut-offs between 2049 and 4096 modes on a multiple of 2048 tokens take the 2048-point kernel in
    # one pass (4 column pairs per workgroup: twice the partial sums, no buffer for the passes' parts);
    # above 8192 modes every kernel needs several passes and the buffer
    m32 = _desc(fc, L=1, H=1, N=32768, d=128, dtype=1)
    part = 2 * 8 * 32768 * 4
    grow = fc.workspace_bytes(m32, 3277, b.FC_PATH_FFT) - fc.workspace_bytes(m32, 1639, b.FC_PATH_FFT)
    assert part <= grow < part + 4096
    assert fc.workspace_bytes(m32, 9000, b.FC_PATH_FFT) >= fc.workspace_bytes(m32, 1639, b.FC_PATH_FFT) + 2 * 32768 * 128 * 4
    # decode attention: group sizes per storage type
    def dec(q_heads, kv_heads, d_, dtype):
        return lib.flashcache_decode_attention(16, 16, 16, 1, 2, kv_heads, q_heads, d_, dtype, 16, 16, 8,
                                               ctypes.c_float(1.0), 16, 256, 1 << 30, None)
    assert dec(34, 2, 128, b.FC_BF16) == b.FC_EUNSUPPORTED      # 17 query heads per KV head
    assert dec(6, 2, 128, b.FC_F32) == b.FC_EUNSUPPORTED        # fp32 caches: groups 1, 2, 4, 7, 8 only
    assert dec(6, 2, 96, b.FC_BF16) == b.FC_EUNSUPPORTED        # head dims 64 and 128 only
    assert dec(5, 2, 128, b.FC_BF16) == b.FC_EINVAL             # q heads not a multiple of kv heads
    # infeasible budgets
    assert lib.flashcache_allocate(16, 1, 4, 2, 64, 3, 1, 64, 16, 16, None) == b.FC_EBUDGET
    assert lib.flashcache_allocate(16, 1, 4, 2, 64, 400, 1, 64, 16, 16, None) == b.FC_EBUDGET
    assert lib.flashcache_allocate(16, 1, 4, 2, 64, 40, 0, 64, 16, 16, None) == b.FC_EBUDGET
    assert lib.flashcache_allocate(16, 1, 4, 2, 64, 40, 1, 65, 16, 16, None) == b.FC_EBUDGET
    assert lib.flashcache_allocate(None, 1, 4, 2, 64, 40, 1, 64, 16, 16, None) == b.FC_EINVAL
    # select_gather: rows_per_seq out of range, null pointers
    assert lib.flashcache_select_gather(16, 16, ref(d), 16, 16, 16, -1, 16, 16, 16, None, 0, None) == b.FC_EINVAL
    assert lib.flashcache_select_gather(16, 16, ref(d), None, 16, 16, 8, 16, 16, 16, None, 0, None) == b.FC_EINVAL
    # empty batch is a successful no-op
    empty = _desc(fc, B=0)
    assert lib.flashcache_score(None, None, ref(empty), 7, 1, None, None, None, 0, None) == b.FC_OK
    assert lib.flashcache_allocate(None, 0, 4, 2, 64, 40, 1, 64, None, None, None) == b.FC_OK
    assert b.status_string(b.FC_EBUDGET).startswith("FC_EBUDGET")
