"""ctypes binding of libflashcache.so: argument marshalling only.

Every step of the path runs in the library's HIP kernels; torch is used for
device memory and for the current stream handle.  There is no fallback: if the
library has not been built, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

# FLASHCACHE_LIBRARY names another build of the same library (bench.py --library sets it for the
# experiment builds of build.py); unset, the product library beside this file is loaded.
_LIB_PATH = os.environ.get("FLASHCACHE_LIBRARY") or os.path.join(
    os.path.dirname(os.path.abspath(__file__)), "libflashcache.so")

FC_OK, FC_EINVAL, FC_EUNSUPPORTED, FC_EWORKSPACE, FC_EBUDGET, FC_EHIP = range(6)
FC_F32, FC_BF16 = 0, 1
FC_PATH_AUTO, FC_PATH_DENSE, FC_PATH_FFT = 0, 1, 2
PATHS = {"auto": FC_PATH_AUTO, "dense": FC_PATH_DENSE, "fft": FC_PATH_FFT}

EXPORTED_SYMBOLS = (
    "flashcache_cutoff_r", "flashcache_total_budget", "flashcache_resolve_path",
    "flashcache_workspace_bytes", "flashcache_select_workspace_bytes", "flashcache_prepare",
    "flashcache_workspace_error", "flashcache_score", "flashcache_score_layer", "flashcache_lowpass_energy",
    "flashcache_allocate",
    "flashcache_select_gather", "flashcache_select_gather_shared", "flashcache_select_gather_paged",
    "flashcache_decode_workspace_bytes", "flashcache_decode_attention",
    "flashcache_decode_attention_paged", "flashcache_decode_static_scratch_bytes",
    "flashcache_decode_attention_static", "flashcache_status_string",
    "flashcache_profile_enable", "flashcache_profile_read",
)


class FcKvDesc(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("layers", ctypes.c_int32), ("kv_heads", ctypes.c_int32),
        ("n_tokens", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("stride_b", ctypes.c_int64), ("stride_l", ctypes.c_int64),
        ("stride_h", ctypes.c_int64), ("stride_n", ctypes.c_int64),
    ]


class FlashCacheError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)}")


def _load() -> ctypes.CDLL:
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is missing: build it first "
            "(python -c 'import __graft_entry__ as g; g.build()'); there is no fallback path")
    lib = ctypes.CDLL(_LIB_PATH)
    c_desc_p = ctypes.POINTER(FcKvDesc)
    vp, i32, i64, sz, dbl = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t, ctypes.c_double
    lib.flashcache_cutoff_r.argtypes, lib.flashcache_cutoff_r.restype = [i32, dbl], i32
    lib.flashcache_total_budget.argtypes, lib.flashcache_total_budget.restype = [i32, i32, dbl], i64
    lib.flashcache_resolve_path.argtypes, lib.flashcache_resolve_path.restype = [c_desc_p, i32, i32], i32
    lib.flashcache_workspace_bytes.argtypes, lib.flashcache_workspace_bytes.restype = [c_desc_p, i32, i32], sz
    lib.flashcache_select_workspace_bytes.argtypes = [c_desc_p]
    lib.flashcache_select_workspace_bytes.restype = sz
    lib.flashcache_prepare.argtypes, lib.flashcache_prepare.restype = [c_desc_p, i32, i32, vp, sz, vp], i32
    lib.flashcache_workspace_error.argtypes = [vp, ctypes.POINTER(i32), vp]
    lib.flashcache_workspace_error.restype = i32
    lib.flashcache_score.argtypes = [vp, vp, c_desc_p, i32, i32, vp, vp, vp, sz, vp]
    lib.flashcache_score_layer.argtypes = [vp, vp, c_desc_p, i32, i32, i32, i32, vp, vp, vp, sz, vp]
    lib.flashcache_score_layer.restype = i32
    lib.flashcache_score.restype = i32
    lib.flashcache_lowpass_energy.argtypes = [c_desc_p, i32, i32, vp, sz, vp, vp]
    lib.flashcache_lowpass_energy.restype = i32
    lib.flashcache_allocate.argtypes = [vp, i32, i32, i32, i32, i64, i32, i32, vp, vp, vp]
    lib.flashcache_allocate.restype = i32
    lib.flashcache_select_gather.argtypes = [vp, vp, c_desc_p, vp, vp, vp, i64, vp, vp, vp, vp, sz, vp]
    lib.flashcache_select_gather.restype = i32
    lib.flashcache_decode_workspace_bytes.argtypes = [i32, i32, i32, i32, i32]
    lib.flashcache_decode_workspace_bytes.restype = sz
    lib.flashcache_decode_attention.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, i32, vp, vp, i64,
                                                ctypes.c_float, vp, vp, sz, vp]
    lib.flashcache_decode_attention.restype = i32
    lib.flashcache_decode_static_scratch_bytes.argtypes = []
    lib.flashcache_decode_static_scratch_bytes.restype = sz
    lib.flashcache_decode_attention_static.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, i32, vp, vp, i64,
                                                       ctypes.c_float, vp, vp]
    lib.flashcache_decode_attention_static.restype = i32
    lib.flashcache_decode_attention_paged.argtypes = [vp, vp, vp, vp, i32, i32, i64, i32, i32, i32, i32, i32, i32,
                                                      vp, ctypes.c_float, vp, vp, sz, vp]
    lib.flashcache_decode_attention_paged.restype = i32
    lib.flashcache_profile_enable.argtypes, lib.flashcache_profile_enable.restype = [i32], i32
    lib.flashcache_profile_read.argtypes = [i32, ctypes.c_char_p, i32, ctypes.POINTER(i32),
                                            ctypes.POINTER(ctypes.c_float), ctypes.POINTER(i32)]
    lib.flashcache_profile_read.restype = i32
    lib.flashcache_select_gather_shared.argtypes = lib.flashcache_select_gather.argtypes
    lib.flashcache_select_gather_shared.restype = i32
    lib.flashcache_select_gather_paged.argtypes = [vp, vp, c_desc_p, vp, vp, vp, i64, i32, vp, vp, i32, i32,
                                                   i64, vp, vp, vp, sz, vp]
    lib.flashcache_select_gather_paged.restype = i32
    lib.flashcache_status_string.argtypes, lib.flashcache_status_string.restype = [i32], ctypes.c_char_p
    return lib


_lib = _load()


def library_path() -> str:
    return _LIB_PATH


def status_string(status: int) -> str:
    return _lib.flashcache_status_string(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != FC_OK:
        raise FlashCacheError(status, where)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def describe(K: torch.Tensor) -> FcKvDesc:
    """Descriptor of a [B, L, H, N, d] tensor (any strides, innermost contiguous)."""
    if K.dim() != 5:
        raise ValueError("K/V must have shape [B, L, H, N, d]")
    if K.stride(4) != 1 and K.shape[4] > 1:
        raise ValueError("the head dimension must be contiguous")
    if K.dtype == torch.float32:
        dt = FC_F32
    elif K.dtype == torch.bfloat16:
        dt = FC_BF16
    else:
        raise ValueError(f"unsupported dtype {K.dtype}")
    B, L, H, N, d = K.shape
    return FcKvDesc(B, L, H, N, d, dt, K.stride(0), K.stride(1), K.stride(2), K.stride(3))


# ---- host helpers ---------------------------------------------------------------------------
def cutoff_r(n_tokens: int, gamma: float) -> int:
    return int(_lib.flashcache_cutoff_r(n_tokens, gamma))


def total_budget(layers: int, n_tokens: int, rho: float) -> int:
    return int(_lib.flashcache_total_budget(layers, n_tokens, rho))


def resolve_path(desc: FcKvDesc, r: int, path: int = FC_PATH_AUTO) -> int:
    return int(_lib.flashcache_resolve_path(ctypes.byref(desc), r, path))


def workspace_bytes(desc: FcKvDesc, r: int, path: int = FC_PATH_AUTO) -> int:
    return int(_lib.flashcache_workspace_bytes(ctypes.byref(desc), r, path))


# ---- device entry points --------------------------------------------------------------------
def prepare(desc: FcKvDesc, r: int, path: int, workspace: torch.Tensor) -> None:
    _check(_lib.flashcache_prepare(ctypes.byref(desc), r, path, _ptr(workspace),
                                   workspace.numel() * workspace.element_size(), _stream()),
           "flashcache_prepare")


def workspace_error(workspace: torch.Tensor) -> int:
    flag = ctypes.c_int32(-1)
    _check(_lib.flashcache_workspace_error(_ptr(workspace), ctypes.byref(flag), _stream()),
           "flashcache_workspace_error")
    return flag.value


def score(K: torch.Tensor, V: torch.Tensor, desc: FcKvDesc, r: int, path: int,
          scores: torch.Tensor, energy: torch.Tensor, workspace: torch.Tensor) -> None:
    _check(_lib.flashcache_score(_ptr(K), _ptr(V), ctypes.byref(desc), r, path, _ptr(scores),
                                 _ptr(energy), _ptr(workspace),
                                 workspace.numel() * workspace.element_size(), _stream()),
           "flashcache_score")


def score_layer(K: torch.Tensor, V: torch.Tensor, desc: FcKvDesc, layer: int, total_layers: int, r: int,
                path: int, scores: torch.Tensor, energy: torch.Tensor, workspace: torch.Tensor) -> None:
    """K, V: one layer of every sequence, [B, 1, H, N, d]; scores / energy: the full
    [B, total_layers, H, N] / [B, total_layers, H, 4] arrays, of which layer `layer` is written."""
    _check(_lib.flashcache_score_layer(_ptr(K), _ptr(V), ctypes.byref(desc), layer, total_layers, r, path,
                                       _ptr(scores), _ptr(energy), _ptr(workspace),
                                       workspace.numel() * workspace.element_size(), _stream()),
           "flashcache_score_layer")


def lowpass_energy(desc: FcKvDesc, r: int, path: int, workspace: torch.Tensor,
                   out: torch.Tensor) -> None:
    """out: float64 [B, L, H, 2]; call right after score() on the same workspace."""
    _check(_lib.flashcache_lowpass_energy(ctypes.byref(desc), r, path, _ptr(workspace),
                                          workspace.numel() * workspace.element_size(), _ptr(out),
                                          _stream()), "flashcache_lowpass_energy")


def allocate(energy: torch.Tensor, batch: int, layers: int, kv_heads: int, n_tokens: int,
             total: int, b_min: int, b_max: int, budgets: torch.Tensor,
             layer_offsets: torch.Tensor) -> None:
    _check(_lib.flashcache_allocate(_ptr(energy), batch, layers, kv_heads, n_tokens, total, b_min,
                                    b_max, _ptr(budgets), _ptr(layer_offsets), _stream()),
           "flashcache_allocate")


def select_gather(K: torch.Tensor, V: torch.Tensor, desc: FcKvDesc, scores: torch.Tensor,
                  budgets: torch.Tensor, layer_offsets: torch.Tensor, rows_per_seq: int,
                  idx_out: torch.Tensor, K_out: torch.Tensor, V_out: torch.Tensor,
                  shared: bool = False) -> None:
    fn = _lib.flashcache_select_gather_shared if shared else _lib.flashcache_select_gather
    _check(fn(_ptr(K), _ptr(V), ctypes.byref(desc), _ptr(scores), _ptr(budgets), _ptr(layer_offsets),
              rows_per_seq, _ptr(idx_out), _ptr(K_out), _ptr(V_out), None, 0, _stream()),
           "flashcache_select_gather_shared" if shared else "flashcache_select_gather")


def select_gather_paged(K: torch.Tensor, V: torch.Tensor, desc: FcKvDesc, scores: torch.Tensor,
                        budgets: torch.Tensor, layer_offsets: torch.Tensor, rows_per_seq: int,
                        idx_out: torch.Tensor, block_table: torch.Tensor, page_size: int,
                        K_cache: torch.Tensor, V_cache: torch.Tensor, shared: bool = False) -> None:
    """block_table int32 [B, L, H, max_pages]; K_cache/V_cache [num_pages, page_size, d]."""
    _check(_lib.flashcache_select_gather_paged(
        _ptr(K), _ptr(V), ctypes.byref(desc), _ptr(scores), _ptr(budgets), _ptr(layer_offsets),
        rows_per_seq, 1 if shared else 0, _ptr(idx_out), _ptr(block_table), page_size,
        block_table.shape[-1], K_cache.shape[0], _ptr(K_cache), _ptr(V_cache), None, 0, _stream()),
        "flashcache_select_gather_paged")


def decode_attention(Q: torch.Tensor, K_cache: torch.Tensor, V_cache: torch.Tensor, kv_heads: int,
                     budgets: torch.Tensor, layer_offsets: torch.Tensor, rows_per_seq: int,
                     scale: float, out: Optional[torch.Tensor] = None,
                     workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Q [B, L, Hq, d]; K_cache/V_cache packed [B, rows_per_seq, d]; returns float32 [B, L, Hq, d]."""
    B, L, Hq, d = Q.shape
    dt = FC_BF16 if Q.dtype == torch.bfloat16 else FC_F32
    need = int(_lib.flashcache_decode_workspace_bytes(B, L, kv_heads, Hq, d))
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=Q.device)
    if out is None:
        out = torch.empty((B, L, Hq, d), dtype=torch.float32, device=Q.device)
    _check(_lib.flashcache_decode_attention(
        _ptr(Q), _ptr(K_cache), _ptr(V_cache), B, L, kv_heads, Hq, d, dt, _ptr(budgets),
        _ptr(layer_offsets), rows_per_seq, scale, _ptr(out), _ptr(workspace),
        workspace.numel(), _stream()), "flashcache_decode_attention")
    return out


def decode_static_scratch_bytes() -> int:
    return int(_lib.flashcache_decode_static_scratch_bytes())


def decode_attention_static(Q: torch.Tensor, K_cache: torch.Tensor, V_cache: torch.Tensor, kv_heads: int,
                            budgets: torch.Tensor, layer_offsets: torch.Tensor, rows_per_seq: int,
                            scale: float, out: torch.Tensor) -> torch.Tensor:
    """decode_attention without a workspace: the library's own fixed scratch array is used and the
    call allocates nothing (`out` must be given: float32 [B, L, Hq, d])."""
    B, L, Hq, d = Q.shape
    dt = FC_BF16 if Q.dtype == torch.bfloat16 else FC_F32
    _check(_lib.flashcache_decode_attention_static(
        _ptr(Q), _ptr(K_cache), _ptr(V_cache), B, L, kv_heads, Hq, d, dt, _ptr(budgets),
        _ptr(layer_offsets), rows_per_seq, scale, _ptr(out), _stream()), "flashcache_decode_attention_static")
    return out


def decode_attention_paged(Q: torch.Tensor, K_pages: torch.Tensor, V_pages: torch.Tensor, kv_heads: int,
                           budgets: torch.Tensor, block_table: torch.Tensor, scale: float,
                           out: Optional[torch.Tensor] = None,
                           workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Q [B, L, Hq, d]; K_pages/V_pages [num_pages, page_size, d]; block_table int32
    [B, L, H, max_pages]; returns float32 [B, L, Hq, d]."""
    B, L, Hq, d = Q.shape
    num_pages, page_size = int(K_pages.shape[0]), int(K_pages.shape[1])
    max_pages = int(block_table.shape[-1])
    dt = FC_BF16 if Q.dtype == torch.bfloat16 else FC_F32
    need = int(_lib.flashcache_decode_workspace_bytes(B, L, kv_heads, Hq, d))
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=Q.device)
    if out is None:
        out = torch.empty((B, L, Hq, d), dtype=torch.float32, device=Q.device)
    _check(_lib.flashcache_decode_attention_paged(
        _ptr(Q), _ptr(K_pages), _ptr(V_pages), _ptr(block_table), page_size, max_pages, num_pages, B, L,
        kv_heads, Hq, d, dt, _ptr(budgets), scale, _ptr(out), _ptr(workspace), workspace.numel(),
        _stream()), "flashcache_decode_attention_paged")
    return out


def profile_enable(on: bool) -> None:
    _check(_lib.flashcache_profile_enable(1 if on else 0), "flashcache_profile_enable")


def profile_read(max_entries: int = 32) -> dict:
    """{kernel name: (launches, total milliseconds)} recorded since profile_enable(True)."""
    stride = 64
    names = ctypes.create_string_buffer(max_entries * stride)
    launches = (ctypes.c_int32 * max_entries)()
    total_ms = (ctypes.c_float * max_entries)()
    n = ctypes.c_int32(0)
    _check(_lib.flashcache_profile_read(max_entries, names, stride, launches, total_ms,
                                        ctypes.byref(n)), "flashcache_profile_read")
    out = {}
    for k in range(min(n.value, max_entries)):
        name = names.raw[k * stride:(k + 1) * stride].split(b"\0", 1)[0].decode()
        out[name] = (int(launches[k]), float(total_ms[k]))
    return out


# ---- convenience: buffers for one shape, and the three calls in order -------------------------
class Compressor:
    """Owns the device buffers for one (shape, r, T) and enqueues score -> allocate -> select_gather.

    Pure plumbing: allocation through torch, then the three C-ABI calls on the current stream.
    """

    def __init__(self, K: torch.Tensor, r: int, total: int, path: str = "auto",
                 b_min: int = 1, b_max: Optional[int] = None, shared: bool = False):
        self.desc = describe(K)
        B, L, H, N, d = K.shape
        self.shape = (B, L, H, N, d)
        self.r, self.total = int(r), int(total)
        self.b_min, self.b_max = int(b_min), int(N if b_max is None else b_max)
        self.shared = bool(shared)
        self.path = resolve_path(self.desc, self.r, PATHS[path])
        if self.path == 0:
            raise FlashCacheError(FC_EUNSUPPORTED, "resolve_path")
        dev = K.device
        nbytes = workspace_bytes(self.desc, self.r, self.path)
        self.workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=dev)
        self.scores = torch.empty((B, L, H, N), dtype=torch.float32, device=dev)
        self.energy = torch.empty((B, L, H, 4), dtype=torch.float64, device=dev)
        self.budgets = torch.empty((B, L), dtype=torch.int32, device=dev)
        self.layer_offsets = torch.empty((B, L + 1), dtype=torch.int64, device=dev)
        self.rows_per_seq = H * self.total
        self.idx = torch.empty((B, self.rows_per_seq), dtype=torch.int32, device=dev)
        self.K_out = torch.empty((B, self.rows_per_seq, d), dtype=K.dtype, device=dev)
        self.V_out = torch.empty((B, self.rows_per_seq, d), dtype=K.dtype, device=dev)
        prepare(self.desc, self.r, self.path, self.workspace)

    def run_score(self, K, V):
        score(K, V, self.desc, self.r, self.path, self.scores, self.energy, self.workspace)

    def run_allocate(self):
        B, L, H, N, _ = self.shape
        allocate(self.energy, B, L, H, N, self.total, self.b_min, self.b_max, self.budgets,
                 self.layer_offsets)

    def run_select_gather(self, K, V):
        select_gather(K, V, self.desc, self.scores, self.budgets, self.layer_offsets,
                      self.rows_per_seq, self.idx, self.K_out, self.V_out, shared=self.shared)

    def run(self, K: torch.Tensor, V: torch.Tensor) -> None:
        self.run_score(K, V)
        self.run_allocate()
        self.run_select_gather(K, V)
