// Decode-step attention over the compacted, per-layer-ragged cache (Preliminary section, Eq. 2-4,
// for one new token per sequence):  out = softmax(q K^T * scale) V  over the b_l rows each
// (layer, KV head) kept.  Grouped-query attention: query head g reads KV head g / G.
//
// HBM-bound by design: every kept K and V row is read exactly once (2*b_l*d*e bytes per unit),
// so the traffic - and the time - shrinks with the retention ratio.  Work is split over rows
// (flash-decoding style): a workgroup streams a chunk of one unit's rows, keeps online-softmax
// states, merges them through LDS and writes (max, sum, weighted V) for its chunk; a second kernel
// merges the chunks.
//
// Two realisations of the chunk kernel:
//  * bf16 caches: the matrix cores (v_mfma_f32_16x16x16_bf16).  With G query heads per KV head the
//    vector ALUs would have to do G dot products and G weighted sums per row and cap the row rate
//    well below HBM speed; as a 16-wide tile of query heads (G <= 16, padded with zeros) the same
//    work is 1.5 matrix instructions per row.  Scores S^T = K Q^T (bf16 x bf16 products are exact
//    in fp32), probabilities in fp32, then P V with P split into two bf16 terms (hi + lo, 16
//    significant bits) so that the weighted sum keeps fp32-grade accuracy.
//  * fp32 caches: vector ALUs, d/8 lanes per row, one online-softmax state per lane group.
#include <mutex>

#include "fc_common.h"

namespace fc {

namespace {

// Scratch of the allocation-free entry point (flashcache_decode_attention_static): the per-chunk
// partial results live in this array instead of a caller workspace.  Every GPU the library runs on
// holds its own copy until the process ends.  In host code the array's name is only a handle: its
// device address is looked up once per device (static_scratch below) and that pointer is what the
// kernels receive.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

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

// Paged source: row j of unit (b,l,h) sits in slot j % page_size of page
// block_table[unit][j / page_size] of caches laid out [num_pages][page_size][d].  table == nullptr
// means the packed layout.  Rows of a page entry that is missing or out of range are not read.
struct PagedSrc {
  const int* table;
  int page_size, max_pages;
  long long num_pages;
};
// cache row index of row `row` of this unit; ok = false (and a readable row) if it has no page
template <bool PAGED>
__device__ __forceinline__ long long cache_row(const PagedSrc& pg, long long packed_base, int unit, int row,
                                               bool& ok) {
  ok = true;
  if (!PAGED) return packed_base + row;
  const int p = row / pg.page_size;
  long long page = -1;
  if (p < pg.max_pages) page = pg.table[(size_t)unit * pg.max_pages + p];
  ok = page >= 0 && page < pg.num_pages;
  return ok ? page * pg.page_size + (row - p * pg.page_size) : 0;
}

template <typename T, int G, int LPR, bool PAGED>
__global__ __launch_bounds__(kDecThreads) void decode_partial_kernel(
    const T* __restrict__ Q, const T* __restrict__ Kc, const T* __restrict__ Vc,
    const int* __restrict__ budgets, const long long* __restrict__ layer_offsets, int L, int H,
    long long rows_per_seq, float scale_log2e, int splits, float* __restrict__ partial, PagedSrc pg) {
  constexpr int D = LPR * 8;
  constexpr int NG = kDecThreads / LPR;                 // lane groups (rows in flight per step / unroll)
  constexpr int NW = kDecThreads / 64;                  // waves; their lane groups merge in registers
  __shared__ float sm_m[NW][G], sm_l[NW][G];
  __shared__ float sm_o[NW][G][D];
  const int split = blockIdx.x, unit = blockIdx.y;
  const int h = unit % H, bl = unit / H, l = bl % L, b = bl / L;
  const int k = budgets[(size_t)b * L + l];
  const long long off = PAGED ? 0 : layer_offsets[(size_t)b * (L + 1) + l] + (long long)h * k;
  float* rec = partial + ((size_t)unit * splits + split) * partial_floats(G, D);
  const int tid = threadIdx.x, grp = tid / LPR, sub = tid % LPR;
  const bool bad = k < 0 || (!PAGED && (off < 0 || off + k > rows_per_seq));
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

  const long long packed_base = PAGED ? 0 : (long long)b * rows_per_seq + off;
  const T* kbase = Kc + sub * 8;
  const T* vbase = Vc + sub * 8;
  for (int row = r0 + grp; row < r1; row += NG * kDecUnroll) {
    float kv[kDecUnroll][8], vv[kDecUnroll][8];
    bool valid[kDecUnroll];
#pragma unroll
    for (int u = 0; u < kDecUnroll; ++u) {
      const int rr = row + u * NG;
      valid[u] = rr < r1;
      const int rc = valid[u] ? rr : row;               // row itself is always in range
      bool ok;
      const long long ci = cache_row<PAGED>(pg, packed_base, unit, rc, ok);
      valid[u] = valid[u] && ok;
      load8<T>(kbase + (size_t)ci * D, kv[u]);
      load8<T>(vbase + (size_t)ci * D, vv[u]);
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
      // mx is finite as soon as one row was valid (packed layout: row `row` always is); while no
      // row has been seen the state stays empty
      if (mx == -INFINITY) continue;
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


// ------------------------------------------------------------------ bf16: matrix-core chunk kernel
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float float4v __attribute__((ext_vector_type(4)));

constexpr int kTilesPerStep = 2;       // 16-row tiles between two rescales of the accumulators

__device__ __forceinline__ short4v as_short4(uint32_t lo, uint32_t hi) {
  union { uint32_t u[2]; short4v v; } c;
  c.u[0] = lo; c.u[1] = hi;
  return c.v;
}
// round-to-nearest-even bf16 bits of a finite float
__device__ __forceinline__ uint32_t bf16_rne(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// Operand layouts of v_mfma_f32_16x16x16_bf16 (D = A B + C, wave of 64 lanes, c16 = lane % 16,
// g4 = lane / 16): A holds row c16, k = 4*g4..4*g4+3; B holds column c16, same k; C/D hold column
// c16, rows 4*g4..4*g4+3.  The order of k inside a product is free as long as A and B agree, which
// lets a lane take its k-values from contiguous bytes of a row:
//   scores:  A = K rows (row c16 of the tile, dims (D/4)*g4 + 4s.. for step s), B = Q (query head
//            c16, same dims)  ->  lane holds S[row 4*g4+i][head c16]
//   output:  A = P (head c16, rows 4*g4+i: exactly the layout the scores come out in), B = V (rows
//            4*g4+i, dim (D/16)*c16 + t for output tile t)  ->  lane holds out[head 4*g4+i][that dim]
template <int D, bool PAGED>
__global__ __launch_bounds__(kDecThreads) void decode_mfma_partial_kernel(
    const uint16_t* __restrict__ Q, const uint16_t* __restrict__ Kc, const uint16_t* __restrict__ Vc,
    const int* __restrict__ budgets, const long long* __restrict__ layer_offsets, int L, int H, int G,
    long long rows_per_seq, float scale_log2e, int splits, float* __restrict__ partial, PagedSrc pg) {
  constexpr int KS = D / 16;            // k-steps of the score product
  constexpr int KW = D / 8;             // dwords of a K row (and of a Q row) per lane: D/4 dims
  constexpr int VT = D / 16;            // output tiles = dims of a V row per lane
  constexpr int VW = VT / 2;            // dwords of a V row per lane
  constexpr int NW = kDecThreads / 64;
  constexpr int GP = 16;                // query heads per tile
  __shared__ float sm_m[NW][GP], sm_l[NW][GP];
  __shared__ float sm_o[NW][GP][D];
  const int split = blockIdx.x, unit = blockIdx.y;
  const int h = unit % H, bl = unit / H, l = bl % L, b = bl / L;
  const int k = budgets[(size_t)b * L + l];
  const long long off = PAGED ? 0 : layer_offsets[(size_t)b * (L + 1) + l] + (long long)h * k;
  float* rec = partial + ((size_t)unit * splits + split) * partial_floats(G, D);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, c16 = lane & 15, g4 = lane >> 4;
  const bool bad = k < 0 || (!PAGED && (off < 0 || off + k > rows_per_seq));
  const int chunk = bad ? 0 : (k + splits - 1) / splits;
  const int r0 = min(k, split * chunk), r1 = bad ? 0 : min(k, r0 + chunk);

  // B operand of the score product: query head c16 (zeros beyond G), dims (D/4)*g4 ..
  uint32_t qw[KW];
#pragma unroll
  for (int i = 0; i < KW; ++i) qw[i] = 0u;
  if (c16 < G) {
    const uint16_t* qp = Q + (((size_t)b * L + l) * ((size_t)H * G) + (size_t)h * G + c16) * D + (D / 4) * g4;
#pragma unroll
    for (int i = 0; i < KW / 4; ++i) {
      const uint4 u = *reinterpret_cast<const uint4*>(qp + 8 * i);
      qw[4 * i] = u.x; qw[4 * i + 1] = u.y; qw[4 * i + 2] = u.z; qw[4 * i + 3] = u.w;
    }
  }

  float m = -INFINITY, ls = 0.f;        // running maximum (common to the 4 lanes of a head) and this lane's sum
  float4v out[VT];
#pragma unroll
  for (int t = 0; t < VT; ++t) out[t] = float4v{0.f, 0.f, 0.f, 0.f};

  const long long packed_base = PAGED ? 0 : (long long)b * rows_per_seq + off;
  const uint16_t* kbase = Kc + (D / 4) * g4;
  const uint16_t* vbase = Vc + VT * c16;
  constexpr int kStepRows = 16 * kTilesPerStep;
  // loads of one step: K rows rb+16*tt+c16, V rows rb+16*tt+4*g4+i (clamped to the chunk; masked later)
  uint32_t kw[kTilesPerStep][KW], vw[kTilesPerStep][4][VW], kwn[kTilesPerStep][KW], vwn[kTilesPerStep][4][VW];
  // vok: bit 4*tt+i set if row rb+16*tt+4*g4+i of the step has a page (always, in the packed layout)
  unsigned vok = ~0u, vokn = ~0u;
  auto load_step = [&](int rb, uint32_t (&kd)[kTilesPerStep][KW], uint32_t (&vd)[kTilesPerStep][4][VW],
                       unsigned& okbits) {
    okbits = 0u;
#pragma unroll
    for (int tt = 0; tt < kTilesPerStep; ++tt) {
      const int kr = min(rb + 16 * tt + c16, r1 - 1);
      bool kok;
      const uint16_t* kp = kbase + (size_t)cache_row<PAGED>(pg, packed_base, unit, kr, kok) * D;
#pragma unroll
      for (int i = 0; i < KW / 4; ++i) {
        const uint4 u = *reinterpret_cast<const uint4*>(kp + 8 * i);
        kd[tt][4 * i] = u.x; kd[tt][4 * i + 1] = u.y; kd[tt][4 * i + 2] = u.z; kd[tt][4 * i + 3] = u.w;
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int vr = min(rb + 16 * tt + 4 * g4 + i, r1 - 1);
        bool ok;
        const uint16_t* vp = vbase + (size_t)cache_row<PAGED>(pg, packed_base, unit, vr, ok) * D;
        okbits |= (ok ? 1u : 0u) << (4 * tt + i);
        if constexpr (VW == 4) {
          const uint4 u = *reinterpret_cast<const uint4*>(vp);
          vd[tt][i][0] = u.x; vd[tt][i][1] = u.y; vd[tt][i][2] = u.z; vd[tt][i][3] = u.w;
        } else {
          const uint2 u = *reinterpret_cast<const uint2*>(vp);
          vd[tt][i][0] = u.x; vd[tt][i][1] = u.y;
        }
      }
    }
  };
  const int rb0 = r0 + wave * kStepRows;
  if (rb0 < r1) load_step(rb0, kw, vw, vok);
  for (int rb = rb0; rb < r1; rb += NW * kStepRows) {
    // the next step's rows travel while this step is computed
    const int rbn = rb + NW * kStepRows;
    if (rbn < r1) load_step(rbn, kwn, vwn, vokn);
    // scores of the step, in log2 units
    float sc[kTilesPerStep][4];
    float mx = -INFINITY;
#pragma unroll
    for (int tt = 0; tt < kTilesPerStep; ++tt) {
      float4v acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s = 0; s < KS; ++s)
        acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(as_short4(kw[tt][2 * s], kw[tt][2 * s + 1]),
                                                        as_short4(qw[2 * s], qw[2 * s + 1]), acc, 0, 0, 0);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const bool valid = rb + 16 * tt + 4 * g4 + i < r1 && ((vok >> (4 * tt + i)) & 1u);
        sc[tt][i] = valid ? acc[i] * scale_log2e : -INFINITY;
        mx = fmaxf(mx, sc[tt][i]);
      }
    }
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    // packed layout: row rb is valid and inputs are finite, so the new maximum is finite; paged
    // layout: a step whose rows all lack a page leaves the state as it is
    const float m_new = fmaxf(m, mx);
    const bool none = m_new == -INFINITY;
    const float alpha = none ? 1.f : exp2f(m - m_new);  // exp2(-inf) = 0 on the first step
    m = m_new;
    float psum = 0.f;
    short4v phi[kTilesPerStep], plo[kTilesPerStep];
#pragma unroll
    for (int tt = 0; tt < kTilesPerStep; ++tt) {
      uint32_t hb[4], lb[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float p = none ? 0.f : exp2f(sc[tt][i] - m_new);
        psum += p;
        const uint32_t pu = __float_as_uint(p);
        hb[i] = pu >> 16;                                // hi = p truncated to bf16
        lb[i] = bf16_rne(p - __uint_as_float(pu & 0xFFFF0000u));
      }
      phi[tt] = as_short4(hb[0] | (hb[1] << 16), hb[2] | (hb[3] << 16));
      plo[tt] = as_short4(lb[0] | (lb[1] << 16), lb[2] | (lb[3] << 16));
    }
    ls = fmaf(ls, alpha, psum);
    // the accumulators hold heads 4*g4+i: fetch their rescale factors from the lanes that own them
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float a_i = __shfl(alpha, 4 * g4 + i, 64);
#pragma unroll
      for (int t = 0; t < VT; ++t) out[t][i] *= a_i;
    }
#pragma unroll
    for (int tt = 0; tt < kTilesPerStep; ++tt) {
#pragma unroll
      for (int t = 0; t < VT; ++t) {
        // element t of the four V rows of this lane: dword t/2, low or high half
        const uint32_t sel = (t & 1) ? 0x07060302u : 0x05040100u;
        const short4v vb = as_short4(__builtin_amdgcn_perm(vw[tt][1][t >> 1], vw[tt][0][t >> 1], sel),
                                     __builtin_amdgcn_perm(vw[tt][3][t >> 1], vw[tt][2][t >> 1], sel));
        out[t] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(phi[tt], vb, out[t], 0, 0, 0);
        out[t] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(plo[tt], vb, out[t], 0, 0, 0);
      }
    }
#pragma unroll
    for (int tt = 0; tt < kTilesPerStep; ++tt) {
#pragma unroll
      for (int i = 0; i < KW; ++i) kw[tt][i] = kwn[tt][i];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < VW; ++j) vw[tt][i][j] = vwn[tt][i][j];
    }
    vok = vokn;
  }

  // the 4 lanes of a head add their sums; then the waves merge through LDS in a fixed order
  ls += __shfl_xor(ls, 16, 64);
  ls += __shfl_xor(ls, 32, 64);
  if (g4 == 0) { sm_m[wave][c16] = m; sm_l[wave][c16] = ls; }
#pragma unroll
  for (int t = 0; t < VT; ++t)
#pragma unroll
    for (int i = 0; i < 4; ++i) sm_o[wave][4 * g4 + i][VT * c16 + t] = out[t][i];
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

// out[unit][g][:] = sum_s o_s w_s / sum_s l_s w_s with w_s = exp2(m_s - max m); zeros if no rows.
// grid = (G, units), one thread per feature.
__global__ void decode_merge_kernel(const float* __restrict__ partial, int G, int d, int splits,
                                    float* __restrict__ out) {
  const int g = blockIdx.x, unit = blockIdx.y, dim = threadIdx.x;
  const size_t stride = partial_floats(G, d);
  const float* base = partial + (size_t)unit * splits * stride;
  float M = -INFINITY;
  for (int s = 0; s < splits; ++s) M = fmaxf(M, base[(size_t)s * stride + g]);
  float acc = 0.f, lt = 0.f;
  if (M > -INFINITY) {
    for (int s = 0; s < splits; ++s) {
      const float* rec = base + (size_t)s * stride;
      const float w = exp2f(rec[g] - M);
      acc = fmaf(rec[2 * G + (size_t)g * d + dim], w, acc);
      lt = fmaf(rec[G + g], w, lt);
    }
  }
  out[((size_t)unit * G + g) * d + dim] = lt > 0.f ? acc / lt : 0.f;
}

int pick_splits(int units) {
  int s = (1024 + units - 1) / units;
  return s < 1 ? 1 : (s > 32 ? 32 : s);
}

template <typename T, int G, int LPR>
hipError_t decode_t(const void* Q, const void* Kc, const void* Vc, int B, int L, int H, const int32_t* budgets,
                    const int64_t* offs, int64_t rows_per_seq, float scale, float* out, float* ws,
                    const PagedSrc& pg, hipStream_t s) {
  const int units = B * L * H, splits = pick_splits(units), d = LPR * 8;
  {
    ProfileScope ps("decode_partial_kernel", s);
    auto launch = [&](auto kern) {
      hipLaunchKernelGGL(kern, dim3(splits, units), dim3(kDecThreads), 0, s, static_cast<const T*>(Q),
                         static_cast<const T*>(Kc), static_cast<const T*>(Vc), budgets,
                         reinterpret_cast<const long long*>(offs), L, H, (long long)rows_per_seq,
                         scale * 1.4426950408889634f, splits, ws, pg);
    };
    if (pg.table) launch(decode_partial_kernel<T, G, LPR, true>);
    else launch(decode_partial_kernel<T, G, LPR, false>);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  ProfileScope ps("decode_merge_kernel", s);
  hipLaunchKernelGGL(decode_merge_kernel, dim3(G, units), dim3(d), 0, s, ws, G, d, splits, out);
  return hipGetLastError();
}

template <int D>
hipError_t decode_mfma_t(const void* Q, const void* Kc, const void* Vc, int B, int L, int H, int G,
                         const int32_t* budgets, const int64_t* offs, int64_t rows_per_seq, float scale,
                         float* out, float* ws, const PagedSrc& pg, hipStream_t s) {
  const int units = B * L * H, splits = pick_splits(units);
  {
    ProfileScope ps("decode_mfma_partial_kernel", s);
    auto launch = [&](auto kern) {
      hipLaunchKernelGGL(kern, dim3(splits, units), dim3(kDecThreads), 0, s, static_cast<const uint16_t*>(Q),
                         static_cast<const uint16_t*>(Kc), static_cast<const uint16_t*>(Vc), budgets,
                         reinterpret_cast<const long long*>(offs), L, H, G, (long long)rows_per_seq,
                         scale * 1.4426950408889634f, splits, ws, pg);
    };
    if (pg.table) launch(decode_mfma_partial_kernel<D, true>);
    else launch(decode_mfma_partial_kernel<D, false>);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  ProfileScope ps("decode_merge_kernel", s);
  hipLaunchKernelGGL(decode_merge_kernel, dim3(G, units), dim3(D), 0, s, ws, G, D, splits, out);
  return hipGetLastError();
}

}  // namespace

bool decode_supported(int group, int d, int dtype) {
  if (d != 64 && d != 128) return false;
  if (dtype == FC_BF16) return group >= 1 && group <= 16;          // matrix-core kernel
  return group == 1 || group == 2 || group == 4 || group == 7 || group == 8;
}

size_t decode_static_scratch_bytes() { return kStaticScratchBytes; }

// Device address of this GPU's copy of `scratch` (looked up on the first call per device, with that
// device current; no allocation).
hipError_t decode_static_scratch(void** ptr) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* addr[kMaxDevices] = {};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (!addr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    addr[dev] = p;
  }
  *ptr = addr[dev];
  return hipSuccess;
}

size_t decode_workspace_bytes(int B, int L, int H, int group, int d) {
  const int units = B * L * H;
  return units == 0 ? 0 : (size_t)units * pick_splits(units) * partial_floats(group, d) * sizeof(float);
}

hipError_t decode_launch(const void* Q, const void* Kc, const void* Vc, int B, int L, int H, int group, int d,
                         int dtype, const int32_t* budgets, const int64_t* offs, int64_t rows_per_seq,
                         float scale, float* out, void* ws, const int32_t* block_table, int32_t page_size,
                         int32_t max_pages, int64_t num_pages, hipStream_t s) {
  float* w = static_cast<float*>(ws);
  const PagedSrc pg{block_table, page_size, max_pages, (long long)num_pages};
  if (dtype == FC_BF16)
    return d == 128
               ? decode_mfma_t<128>(Q, Kc, Vc, B, L, H, group, budgets, offs, rows_per_seq, scale, out, w, pg, s)
               : decode_mfma_t<64>(Q, Kc, Vc, B, L, H, group, budgets, offs, rows_per_seq, scale, out, w, pg, s);
#define FC_DEC(GV)                                                                                          \
  if (group == GV)                                                                                          \
    return d == 128                                                                                         \
               ? decode_t<float, GV, 16>(Q, Kc, Vc, B, L, H, budgets, offs, rows_per_seq, scale, out, w, pg, s) \
               : decode_t<float, GV, 8>(Q, Kc, Vc, B, L, H, budgets, offs, rows_per_seq, scale, out, w, pg, s);
  FC_DEC(1) FC_DEC(2) FC_DEC(4) FC_DEC(7) FC_DEC(8)
#undef FC_DEC
  return hipErrorInvalidValue;
}

}  // namespace fc
