// Decode-step attention over the compacted, per-layer-ragged cache (Preliminary section, Eq. 2-4,
// for one new token per sequence):  out = softmax(q K^T * scale) V  over the b_l rows each
// (layer, KV head) kept.  Grouped-query attention: query head g reads KV head g / G.
//
// HBM-bound by design: every kept K and V row is read exactly once (2*b_l*d*e bytes per unit),
// so the traffic - and the time - shrinks with the retention ratio.  Work is split over rows
// (flash-decoding style): a workgroup streams a chunk of one unit's rows with 16-byte loads,
// d/8 lanes per row, keeps one online-softmax state per lane group, merges the groups through
// LDS and writes (max, sum, weighted V) for its chunk; a second kernel merges the chunks.
// All arithmetic is fp32 on exactly-widened inputs.
#include "fc_common.h"

namespace fc {

namespace {

constexpr int kDecThreads = 256;
constexpr int kDecUnroll = 4;          // rows per lane group and step
constexpr int kQuadXor1 = 0xB1, kQuadXor2 = 0x4E, kRowHalfMirror = 0x141, kRowMirror = 0x140;

template <int CTRL> __device__ __forceinline__ float dpp_add(float v) {
  return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
// sum over the LPR (8 or 16) adjacent lanes that share a row; every lane gets the sum
template <int LPR> __device__ __forceinline__ float row_sum(float v) {
  v = dpp_add<kQuadXor1>(v);
  v = dpp_add<kQuadXor2>(v);
  v = dpp_add<kRowHalfMirror>(v);
  if (LPR == 16) v = dpp_add<kRowMirror>(v);
  return v;
}

template <typename T> __device__ __forceinline__ void load8(const T* p, float (&o)[8]);
template <> __device__ __forceinline__ void load8<uint16_t>(const uint16_t* p, float (&o)[8]) {
  const uint4 q = *reinterpret_cast<const uint4*>(p);
  o[0] = __uint_as_float(q.x << 16); o[1] = __uint_as_float(q.x & 0xFFFF0000u);
  o[2] = __uint_as_float(q.y << 16); o[3] = __uint_as_float(q.y & 0xFFFF0000u);
  o[4] = __uint_as_float(q.z << 16); o[5] = __uint_as_float(q.z & 0xFFFF0000u);
  o[6] = __uint_as_float(q.w << 16); o[7] = __uint_as_float(q.w & 0xFFFF0000u);
}
template <> __device__ __forceinline__ void load8<float>(const float* p, float (&o)[8]) {
  const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
  o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w; o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
}

// partial record of one (unit, split): m[G], l[G], o[G][d]  (floats)
__host__ __device__ inline size_t partial_floats(int G, int d) { return (size_t)G * (d + 2); }

template <typename T, int G, int LPR>
__global__ __launch_bounds__(kDecThreads) void decode_partial_kernel(
    const T* __restrict__ Q, const T* __restrict__ Kc, const T* __restrict__ Vc,
    const int* __restrict__ budgets, const long long* __restrict__ layer_offsets, int L, int H,
    long long rows_per_seq, float scale_log2e, int splits, float* __restrict__ partial) {
  constexpr int D = LPR * 8;
  constexpr int NG = kDecThreads / LPR;                 // lane groups (rows in flight per step / unroll)
  constexpr int NW = kDecThreads / 64;                  // waves; their lane groups merge in registers
  __shared__ float sm_m[NW][G], sm_l[NW][G];
  __shared__ float sm_o[NW][G][D];
  const int split = blockIdx.x, unit = blockIdx.y;
  const int h = unit % H, bl = unit / H, l = bl % L, b = bl / L;
  const int k = budgets[(size_t)b * L + l];
  const long long off = layer_offsets[(size_t)b * (L + 1) + l] + (long long)h * k;
  float* rec = partial + ((size_t)unit * splits + split) * partial_floats(G, D);
  const int tid = threadIdx.x, grp = tid / LPR, sub = tid % LPR;
  const bool bad = k < 0 || off < 0 || off + k > rows_per_seq;
  const int chunk = bad ? 0 : (k + splits - 1) / splits;
  const int r0 = min(k, split * chunk), r1 = bad ? 0 : min(k, r0 + chunk);

  // this lane's 8 dims of the G query vectors, pre-multiplied by scale*log2(e)
  float q[G][8];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    load8<T>(Q + (((size_t)b * L + l) * (H * G) + (size_t)h * G + g) * D + sub * 8, q[g]);
#pragma unroll
    for (int i = 0; i < 8; ++i) q[g][i] *= scale_log2e;
  }
  float m[G], ls[G], o[G][8];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m[g] = -INFINITY; ls[g] = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) o[g][i] = 0.f;
  }

  const T* kbase = Kc + ((size_t)b * rows_per_seq + off) * D + sub * 8;
  const T* vbase = Vc + ((size_t)b * rows_per_seq + off) * D + sub * 8;
  for (int row = r0 + grp; row < r1; row += NG * kDecUnroll) {
    float kv[kDecUnroll][8], vv[kDecUnroll][8];
    bool valid[kDecUnroll];
#pragma unroll
    for (int u = 0; u < kDecUnroll; ++u) {
      const int rr = row + u * NG;
      valid[u] = rr < r1;
      const int rc = valid[u] ? rr : row;               // row itself is always in range
      load8<T>(kbase + (size_t)rc * D, kv[u]);
      load8<T>(vbase + (size_t)rc * D, vv[u]);
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float s[kDecUnroll];
      float mx = m[g];
#pragma unroll
      for (int u = 0; u < kDecUnroll; ++u) {
        float acc = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) acc = fmaf(q[g][i], kv[u][i], acc);
        acc = row_sum<LPR>(acc);
        s[u] = valid[u] ? acc : -INFINITY;
        mx = fmaxf(mx, s[u]);
      }
      // mx is finite: row `row` is valid and inputs are finite
      const float alpha = exp2f(m[g] - mx);             // exp2(-inf) = 0 on the first step
      float psum = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) o[g][i] *= alpha;
#pragma unroll
      for (int u = 0; u < kDecUnroll; ++u) {
        const float p = exp2f(s[u] - mx);
        psum += p;
#pragma unroll
        for (int i = 0; i < 8; ++i) o[g][i] = fmaf(p, vv[u][i], o[g][i]);
      }
      ls[g] = fmaf(ls[g], alpha, psum);
      m[g] = mx;
    }
  }

  // merge the lane groups of a wave (lanes that hold the same dims of different rows), then the
  // waves through LDS; the order of the merges is fixed
#pragma unroll
  for (int off = LPR; off < 64; off <<= 1) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float m2 = __shfl_xor(m[g], off, 64), l2 = __shfl_xor(ls[g], off, 64);
      const float M = fmaxf(m[g], m2);
      const float w1 = M > -INFINITY ? exp2f(m[g] - M) : 0.f, w2 = M > -INFINITY ? exp2f(m2 - M) : 0.f;
      ls[g] = ls[g] * w1 + l2 * w2;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float o2 = __shfl_xor(o[g][i], off, 64);
        o[g][i] = o[g][i] * w1 + o2 * w2;
      }
      m[g] = M;
    }
  }
  const int wave = tid >> 6;
  if ((tid & 63) < LPR) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      if (sub == 0) { sm_m[wave][g] = m[g]; sm_l[wave][g] = ls[g]; }
#pragma unroll
      for (int i = 0; i < 8; ++i) sm_o[wave][g][sub * 8 + i] = o[g][i];
    }
  }
  __syncthreads();
  for (int item = tid; item < G * D; item += kDecThreads) {
    const int g = item / D, dim = item % D;
    float M = -INFINITY;
    for (int s2 = 0; s2 < NW; ++s2) M = fmaxf(M, sm_m[s2][g]);
    float acc = 0.f, lt = 0.f;
    if (M > -INFINITY) {
      for (int s2 = 0; s2 < NW; ++s2) {
        const float w = exp2f(sm_m[s2][g] - M);
        acc = fmaf(sm_o[s2][g][dim], w, acc);
        lt = fmaf(sm_l[s2][g], w, lt);
      }
    }
    rec[2 * G + (size_t)g * D + dim] = acc;
    if (dim == 0) { rec[g] = M; rec[G + g] = lt; }
  }
}

// out[unit][g][:] = sum_s o_s w_s / sum_s l_s w_s with w_s = exp2(m_s - max m); zeros if no rows
template <int G>
__global__ __launch_bounds__(kDecThreads) void decode_merge_kernel(const float* __restrict__ partial, int d,
                                                                  int splits, float* __restrict__ out) {
  const int unit = blockIdx.x;
  const float* base = partial + (size_t)unit * splits * partial_floats(G, d);
  for (int item = threadIdx.x; item < G * d; item += kDecThreads) {
    const int g = item / d, dim = item % d;
    float M = -INFINITY;
    for (int s = 0; s < splits; ++s) M = fmaxf(M, base[(size_t)s * partial_floats(G, d) + g]);
    float acc = 0.f, lt = 0.f;
    if (M > -INFINITY) {
      for (int s = 0; s < splits; ++s) {
        const float* rec = base + (size_t)s * partial_floats(G, d);
        const float w = exp2f(rec[g] - M);
        acc = fmaf(rec[2 * G + (size_t)g * d + dim], w, acc);
        lt = fmaf(rec[G + g], w, lt);
      }
    }
    out[((size_t)unit * G + g) * d + dim] = lt > 0.f ? acc / lt : 0.f;
  }
}

int pick_splits(int units) {
  int s = (1024 + units - 1) / units;
  return s < 1 ? 1 : (s > 32 ? 32 : s);
}

template <typename T, int G, int LPR>
hipError_t decode_t(const void* Q, const void* Kc, const void* Vc, int B, int L, int H, const int32_t* budgets,
                    const int64_t* offs, int64_t rows_per_seq, float scale, float* out, float* ws,
                    hipStream_t s) {
  const int units = B * L * H, splits = pick_splits(units), d = LPR * 8;
  {
    ProfileScope ps("decode_partial_kernel", s);
    hipLaunchKernelGGL((decode_partial_kernel<T, G, LPR>), dim3(splits, units), dim3(kDecThreads), 0, s,
                       static_cast<const T*>(Q), static_cast<const T*>(Kc), static_cast<const T*>(Vc),
                       budgets, reinterpret_cast<const long long*>(offs), L, H, (long long)rows_per_seq,
                       scale * 1.4426950408889634f, splits, ws);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  ProfileScope ps("decode_merge_kernel", s);
  hipLaunchKernelGGL(decode_merge_kernel<G>, dim3(units), dim3(kDecThreads), 0, s, ws, d, splits, out);
  return hipGetLastError();
}

}  // namespace

bool decode_supported(int group, int d) { return (d == 64 || d == 128) && (group == 1 || group == 2 ||
                                                 group == 4 || group == 7 || group == 8); }

size_t decode_workspace_bytes(int B, int L, int H, int group, int d) {
  const int units = B * L * H;
  return units == 0 ? 0 : (size_t)units * pick_splits(units) * partial_floats(group, d) * sizeof(float);
}

hipError_t decode_launch(const void* Q, const void* Kc, const void* Vc, int B, int L, int H, int group, int d,
                         int dtype, const int32_t* budgets, const int64_t* offs, int64_t rows_per_seq,
                         float scale, float* out, void* ws, hipStream_t s) {
  float* w = static_cast<float*>(ws);
#define FC_DEC(GV)                                                                                          \
  if (group == GV) {                                                                                        \
    if (dtype == FC_BF16)                                                                                   \
      return d == 128 ? decode_t<uint16_t, GV, 16>(Q, Kc, Vc, B, L, H, budgets, offs, rows_per_seq, scale, out, w, s) \
                      : decode_t<uint16_t, GV, 8>(Q, Kc, Vc, B, L, H, budgets, offs, rows_per_seq, scale, out, w, s); \
    return d == 128 ? decode_t<float, GV, 16>(Q, Kc, Vc, B, L, H, budgets, offs, rows_per_seq, scale, out, w, s)     \
                    : decode_t<float, GV, 8>(Q, Kc, Vc, B, L, H, budgets, offs, rows_per_seq, scale, out, w, s);     \
  }
  FC_DEC(1) FC_DEC(2) FC_DEC(4) FC_DEC(7) FC_DEC(8)
#undef FC_DEC
  return hipErrorInvalidValue;
}

}  // namespace fc
