// Shared declarations of the library's translation units (host side + small device helpers).
#ifndef FC_COMMON_H_
#define FC_COMMON_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "flashcache.h"

namespace fc {

constexpr uint32_t kWsMagic = 0xFC5C0DE1u;
constexpr size_t kWsAlign = 256;

// First 256 bytes of every score workspace, written by flashcache_prepare.
struct WsHeader {
  uint32_t magic;
  int32_t path, n, r, d, dtype;
  int32_t error;        // raised by kernels that find a header not matching their arguments
  int32_t reserved[57];
};
static_assert(sizeof(WsHeader) == 256, "header is one 256-byte slot");

struct KvStrides {
  int64_t sb, sl, sh, sn;  // elements
  int32_t L, H;
};

// Offsets (bytes from the workspace base) of the regions of the dense realisation.
struct DenseLayout {
  int32_t re_pad, r_pad, n_pad, splits, tok_per_split, tiles;   // even-mode columns; all columns; folded rows
  size_t basis, coeff, epart, total;
};
// ... and of the fast-transform realisation.
struct FftLayout {
  int32_t slabs, tiles, passes;   // column groups per tensor; finalize workgroups per unit; passes
  int32_t lane_radix;             // 16, 8, 4, 2 or 1: the register-resident transform has 256*lane_radix points
  size_t twiddle, phase, partial, etot, epart, resid, total;
};

DenseLayout dense_layout(const fc_kv_desc& d, int32_t r);
bool fft_supported(const fc_kv_desc& d, int32_t r);
FftLayout fft_layout(const fc_kv_desc& d, int32_t r);

// launchers (each returns hipGetLastError() after enqueueing)
hipError_t dense_prepare(const fc_kv_desc& d, int32_t r, const DenseLayout& lay, void* ws, hipStream_t s);
// Where a unit's scores and energies go: identity (L = 0), or layer `l` of full arrays
// [B][L][H][..] when the call covers one layer of every sequence (layer-by-layer scoring).
struct UnitMap { int32_t H, L, l; };
__host__ __device__ inline int64_t out_unit(const UnitMap& m, int u) {
  return m.L ? ((int64_t)(u / m.H) * m.L + m.l) * m.H + (u % m.H) : (int64_t)u;
}
hipError_t dense_score(const void* K, const void* V, const fc_kv_desc& d, int32_t r,
                       const DenseLayout& lay, float* scores, double* energy, void* ws, UnitMap um,
                       hipStream_t s);
hipError_t dense_lowpass(const fc_kv_desc& d, const DenseLayout& lay, void* ws, double* lowpass, hipStream_t s);
hipError_t fft_lowpass(const fc_kv_desc& d, int32_t r, const FftLayout& lay, void* ws, double* lowpass,
                       hipStream_t s);
hipError_t fft_prepare(const fc_kv_desc& d, int32_t r, const FftLayout& lay, void* ws, hipStream_t s);
// One pass of the transform kernel; one entry per lane radix (each compiled in its own unit).
struct FftPassArgs {
  const void* K; const void* V; KvStrides st;
  int n, n2, r, rcut, cmode, d, dtype, q0, nbuf, n_ut, slabs;
  WsHeader* hdr; const float2* twn; const float2* phase; float* partial; double* etot; float* resid;
};
hipError_t fft_launch_pass_r16(const FftPassArgs& a, int cp, int q, int mode, hipStream_t s);
hipError_t fft_launch_pass_r8(const FftPassArgs& a, int cp, int q, int mode, hipStream_t s);
hipError_t fft_launch_pass_r4(const FftPassArgs& a, int cp, int q, int mode, hipStream_t s);
hipError_t fft_launch_pass_r2(const FftPassArgs& a, int cp, int q, int mode, hipStream_t s);
hipError_t fft_launch_pass_r1(const FftPassArgs& a, int cp, int q, int mode, hipStream_t s);
hipError_t fft_score(const void* K, const void* V, const fc_kv_desc& d, int32_t r,
                     const FftLayout& lay, float* scores, double* energy, void* ws, UnitMap um,
                     hipStream_t s);
// energy[u][0..3] = sum over tiles of epart[u][tile][0..3], fixed order
hipError_t energy_reduce_launch(const double* epart, int tiles, int units, double* energy, UnitMap um,
                                hipStream_t s);
hipError_t allocate_launch(const double* energy, int32_t B, int32_t L, int32_t H, int32_t N,
                           int64_t T, int32_t b_min, int32_t b_max, int32_t* budgets,
                           int64_t* layer_offsets, hipStream_t s);
hipError_t select_gather_launch(const void* K, const void* V, const fc_kv_desc& d,
                                const float* scores, const int32_t* budgets,
                                const int64_t* layer_offsets, int64_t rows_per_seq, bool shared,
                                int32_t* idx_out, void* K_out, void* V_out, const int32_t* block_table,
                                int32_t page_size, int32_t max_pages, int64_t num_pages, hipStream_t s);

bool decode_supported(int group, int d, int dtype);
size_t decode_workspace_bytes(int B, int L, int H, int group, int d);
size_t decode_static_scratch_bytes();
hipError_t decode_static_scratch(void** ptr);
hipError_t decode_launch(const void* Q, const void* Kc, const void* Vc, int B, int L, int H, int group, int d,
                         int dtype, const int32_t* budgets, const int64_t* offs, int64_t rows_per_seq,
                         float scale, float* out, void* ws, const int32_t* block_table, int32_t page_size,
                         int32_t max_pages, int64_t num_pages, hipStream_t s);

// Per-kernel event timing (see profile.hip): brackets the launches made while it is alive.
bool profiling_on();
class ProfileScope {
 public:
  ProfileScope(const char* name, hipStream_t s);
  ~ProfileScope();
 private:
  hipStream_t stream_;
  long idx_;
};

inline KvStrides strides_of(const fc_kv_desc& d) {
  return KvStrides{d.stride_b, d.stride_l, d.stride_h, d.stride_n, d.layers, d.kv_heads};
}

#if defined(__HIPCC__)
__device__ __forceinline__ float bf16_to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

// True (and raises the flag once) if the workspace was not prepared for these arguments.
__device__ __forceinline__ bool ws_mismatch(WsHeader* h, int path, int n, int r, int d, int dtype) {
  bool bad = h->magic != kWsMagic || h->path != path || h->n != n || h->r != r || h->d != d ||
             h->dtype != dtype;
  if (bad && threadIdx.x == 0) h->error = 1;
  return bad;
}

// Base element offset of unit u = (b*L + l)*H + h.
__device__ __forceinline__ int64_t unit_offset(const KvStrides& st, int u) {
  int h = u % st.H;
  int bl = u / st.H;
  int l = bl % st.L;
  int b = bl / st.L;
  return (int64_t)b * st.sb + (int64_t)l * st.sl + (int64_t)h * st.sh;
}
#endif

}  // namespace fc
#endif
