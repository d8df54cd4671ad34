// Dense realisation of the low-pass projection (Eq. 6-10) on the fp32 matrix cores.
//
//   basis[i][m] = alpha[m] * cos(pi * m * (2i+1) / (2N))          (Eq. 7), fp64 -> fp32 table
//   coeff       = basis^T X            r x d per tensor            (Eq. 6, rows m < r only: Eq. 8)
//   base        = basis coeff          N x d                       (Eq. 9)
//   score[x]    = mean_c (K-K_base)^2 + mean_c (V-V_base)^2        (Eq. 10)
//
// Both products run on v_mfma_f32_32x32x2_f32 (fp32 in, fp32 accumulate).  Works for any N; the
// cost grows like r*N*d, so it is the realisation of choice only for small r or for token counts
// the fast transform does not cover.
//
// The cosine of Eq. 7 satisfies basis[N-1-i][m] = (-1)^m basis[i][m], which halves both products:
// with nh = ceil(N/2), xs[i] = x[i] + x[N-1-i] and xa[i] = x[i] - x[N-1-i] (i < nh; the middle token
// of an odd N counts once in xs and not at all in xa),
//   coeff[even m] = sum_{i<nh} basis[i][m] xs[i],     coeff[odd m] = sum_{i<nh} basis[i][m] xa[i],
//   base[i] = E[i] + O[i],  base[N-1-i] = E[i] - O[i],   E / O = sums over the even / odd modes.
// The table holds only rows i < nh, with the even modes first (columns [0, re_pad)) and the odd
// modes after them (columns [re_pad, r_pad)); the coefficient arrays use the same column order.
#include "fc_common.h"

namespace fc {

typedef float floatx16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int kMTile = 64;   // coefficient rows per workgroup (forward) / chunk of modes (inverse: 32)
constexpr int kTokChunk = 32;
constexpr int kTokTile = 64; // tokens per workgroup in the scoring kernel

// ------------------------------------------------------------------ basis table (step A1)
__global__ void dense_basis_kernel(WsHeader* hdr, float* __restrict__ basis, int n, int r, int re_pad,
                                   int r_pad, int n_pad, int d, int dtype) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx == 0) {
    hdr->magic = kWsMagic; hdr->path = FC_PATH_DENSE; hdr->n = n; hdr->r = r; hdr->d = d;
    hdr->dtype = dtype; hdr->error = 0;
  }
  int64_t total = (int64_t)n_pad * r_pad;
  if (idx >= total) return;
  const int i = (int)(idx / r_pad), col = (int)(idx % r_pad);
  const int m = col < re_pad ? 2 * col : 2 * (col - re_pad) + 1;
  const int nh = (n + 1) / 2;
  float v = 0.f;
  if (i < nh && m < r) {
    // exact integer reduction of m*(2i+1) modulo the period 4N, then one cosine in fp64
    int64_t k = ((int64_t)m * (2 * (int64_t)i + 1)) % (4 * (int64_t)n);
    double alpha = (m == 0) ? sqrt(1.0 / (double)n) : sqrt(2.0 / (double)n);
    v = (float)(alpha * cospi((double)k / (2.0 * (double)n)));
  }
  basis[idx] = v;
}

// ------------------------------------------------------------------ tile loads
// Writes rows [t0, t0+rows) of xs (odd = false) or xa (odd = true) as fp32 into LDS; zeros past nh
// and in the columns [d_act, d) that pad the head dimension to the kernels' multiple of 64.
template <typename T>
__device__ __forceinline__ void load_x_tile(const T* __restrict__ x, int64_t sn, int n, int t0, int rows,
                                            int d, float* __restrict__ xs, int ld, bool odd, int d_act);

template <>
__device__ __forceinline__ void load_x_tile<uint16_t>(const uint16_t* __restrict__ x, int64_t sn, int n,
                                                      int t0, int rows, int d, float* __restrict__ xs,
                                                      int ld, bool odd, int d_act) {
  const int vec_per_row = d / 8, nh = (n + 1) / 2;
  const float sg = odd ? -1.f : 1.f;
  for (int v = threadIdx.x; v < rows * vec_per_row; v += blockDim.x) {
    const int row = v / vec_per_row, c8 = (v % vec_per_row) * 8;
    const int t = t0 + row, tm = n - 1 - t;
    uint4 q = make_uint4(0, 0, 0, 0), p = make_uint4(0, 0, 0, 0);
    float w = 0.f;                          // weight of the row itself: 0 for the middle token in xa
    if (t < nh && c8 < d_act) {
      q = *reinterpret_cast<const uint4*>(x + (int64_t)t * sn + c8);
      w = (tm == t && odd) ? 0.f : 1.f;
      if (tm != t) p = *reinterpret_cast<const uint4*>(x + (int64_t)tm * sn + c8);
    }
    float* o = xs + row * ld + c8;
    const uint32_t qa[4] = {q.x, q.y, q.z, q.w}, pa[4] = {p.x, p.y, p.z, p.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      o[2 * e] = fmaf(sg, bf16_to_f32(pa[e] & 0xFFFFu), w * bf16_to_f32(qa[e] & 0xFFFFu));
      o[2 * e + 1] = fmaf(sg, bf16_to_f32(pa[e] >> 16), w * bf16_to_f32(qa[e] >> 16));
    }
  }
}

template <>
__device__ __forceinline__ void load_x_tile<float>(const float* __restrict__ x, int64_t sn, int n, int t0,
                                                   int rows, int d, float* __restrict__ xs, int ld,
                                                   bool odd, int d_act) {
  const int vec_per_row = d / 4, nh = (n + 1) / 2;
  const float sg = odd ? -1.f : 1.f;
  for (int v = threadIdx.x; v < rows * vec_per_row; v += blockDim.x) {
    const int row = v / vec_per_row, c4 = (v % vec_per_row) * 4;
    const int t = t0 + row, tm = n - 1 - t;
    float4 q = make_float4(0.f, 0.f, 0.f, 0.f), p = q;
    float w = 0.f;
    if (t < nh && c4 < d_act) {
      q = *reinterpret_cast<const float4*>(x + (int64_t)t * sn + c4);
      w = (tm == t && odd) ? 0.f : 1.f;
      if (tm != t) p = *reinterpret_cast<const float4*>(x + (int64_t)tm * sn + c4);
    }
    *reinterpret_cast<float4*>(xs + row * ld + c4) =
        make_float4(fmaf(sg, p.x, w * q.x), fmaf(sg, p.y, w * q.y), fmaf(sg, p.z, w * q.z),
                    fmaf(sg, p.w, w * q.w));
  }
}

template <typename T> __device__ __forceinline__ float load_elem(const T* p);
template <> __device__ __forceinline__ float load_elem<uint16_t>(const uint16_t* p) { return bf16_to_f32(*p); }
template <> __device__ __forceinline__ float load_elem<float>(const float* p) { return *p; }

// ------------------------------------------------------------------ forward: coeff = basis^T X
// grid = (r_pad/64, splits, 2*units), tokens i < n_pad (the folded half); 256 threads = 4 waves; wave w owns coefficient rows
// (w&1)*32.. and columns (w>>1)*(d/2).., i.e. TPW = d/64 accumulator tiles of 32x32.
template <typename T, int TPW>
__global__ __launch_bounds__(256) void dense_coeff_kernel(
    const T* __restrict__ K, const T* __restrict__ V, KvStrides st, int n, int r, int re_pad, int r_pad,
    int n_pad, int tok_per_split, int splits, WsHeader* hdr, const float* __restrict__ basis,
    float* __restrict__ coeff, int dtype, int d) {
  constexpr int D = TPW * 64;               // head dimension padded to a multiple of 64 (pad columns are zero)
  if (ws_mismatch(hdr, FC_PATH_DENSE, n, r, d, dtype)) return;
  __shared__ float Bs[kTokChunk][kMTile];
  __shared__ float Xs[kTokChunk][D];
  const int mtile = blockIdx.x, split = blockIdx.y, u2 = blockIdx.z;
  const int unit = u2 >> 1, tensor = u2 & 1;
  const bool odd = mtile * kMTile >= re_pad;     // this tile's columns are odd modes: they see xa
  const T* x = (tensor ? V : K) + unit_offset(st, unit);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int mb = wave & 1, cw = wave >> 1;
  const int l32 = lane & 31, lhi = lane >> 5;

  floatx16 acc[TPW];
#pragma unroll
  for (int j = 0; j < TPW; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;

  const int t_begin = split * tok_per_split;
  const int t_end = min(n_pad, t_begin + tok_per_split);
  for (int t0 = t_begin; t0 < t_end; t0 += kTokChunk) {
    for (int v = threadIdx.x; v < kTokChunk * kMTile / 4; v += 256) {
      int row = v / (kMTile / 4), c4 = (v % (kMTile / 4)) * 4;
      *reinterpret_cast<float4*>(&Bs[row][c4]) =
          *reinterpret_cast<const float4*>(basis + (int64_t)(t0 + row) * r_pad + mtile * kMTile + c4);
    }
    load_x_tile<T>(x, st.sn, n, t0, kTokChunk, D, &Xs[0][0], D, odd, d);
    __syncthreads();
    // operands of step k+1 are read from LDS while the matrix cores work on step k
    float a_op[2], b_op[2][TPW];
    a_op[0] = Bs[lhi][mb * 32 + l32];
#pragma unroll
    for (int j = 0; j < TPW; ++j) b_op[0][j] = Xs[lhi][cw * (D / 2) + j * 32 + l32];
#pragma unroll
    for (int kk = 0; kk < kTokChunk / 2; ++kk) {
      const int cur = kk & 1, nxt = cur ^ 1;
      if (kk + 1 < kTokChunk / 2) {
        a_op[nxt] = Bs[2 * (kk + 1) + lhi][mb * 32 + l32];
#pragma unroll
        for (int j = 0; j < TPW; ++j) b_op[nxt][j] = Xs[2 * (kk + 1) + lhi][cw * (D / 2) + j * 32 + l32];
      }
      __builtin_amdgcn_sched_barrier(0);    // keep the reads ahead of the products they overlap with
#pragma unroll
      for (int j = 0; j < TPW; ++j)
        acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_op[cur], b_op[cur][j], acc[j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    __syncthreads();
  }
  float* out = coeff + ((int64_t)u2 * splits + split) * r_pad * D;
#pragma unroll
  for (int j = 0; j < TPW; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      int row = mtile * kMTile + mb * 32 + 8 * (i >> 2) + 4 * lhi + (i & 3);
      int col = cw * (D / 2) + j * 32 + l32;
      out[(int64_t)row * D + col] = acc[j][i];
    }
}

// ------------------------------------------------------------------ inverse + fused scoring
// grid = (n_pad/64, units) over the folded half i < nh; wave w owns rows (w&1)*32.. and columns
// (w>>1)*(d/2)...  Each row i yields the scores of tokens i and N-1-i.
template <typename T, int TPW>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(TPW <= 2 ? 3 : 2))) void dense_score_kernel(
    const T* __restrict__ K, const T* __restrict__ V, KvStrides st, int n, int r, int re_pad, int r_pad,
    int splits, WsHeader* hdr, const float* __restrict__ basis, const float* __restrict__ coeff,
    float* __restrict__ scores, double* __restrict__ epart, int tiles, int dtype, int d, UnitMap um) {
  constexpr int D = TPW * 64;               // padded head dimension; columns >= d hold zeros
  if (ws_mismatch(hdr, FC_PATH_DENSE, n, r, d, dtype)) return;
  __shared__ float Bs[kTokTile][33];
  __shared__ float Cs[32][D];
  __shared__ float red[2][4][2][kTokTile];  // [tensor][hp, tot of token i | of token N-1-i][column half][row]
  const int tile = blockIdx.x, unit = blockIdx.y;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int tb = wave & 1, cw = wave >> 1;
  const int l32 = lane & 31, lhi = lane >> 5;
  const int64_t uoff = unit_offset(st, unit);
  const int nh = (n + 1) / 2;

  for (int tensor = 0; tensor < 2; ++tensor) {
    const T* x = (tensor ? V : K) + uoff;
    const float* cf = coeff + (int64_t)(unit * 2 + tensor) * splits * r_pad * D;
    floatx16 acc_e[TPW], acc_o[TPW];
#pragma unroll
    for (int j = 0; j < TPW; ++j)
#pragma unroll
      for (int i = 0; i < 16; ++i) { acc_e[j][i] = 0.f; acc_o[j][i] = 0.f; }

    // columns [0, re_pad) are even modes (accumulate E), the rest odd modes (accumulate O)
    floatx16 acc[TPW];
#pragma unroll
    for (int j = 0; j < TPW; ++j)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
    // the next chunk of the table and of the coefficients travels in registers while the matrix
    // cores work on the current one
    constexpr int NB = kTokTile * 32 / 4 / 256, NC = 32 * D / 4 / 256;
    float4 pb[NB], pc[NC];
    auto fetch = [&](int m0) {
#pragma unroll
      for (int q = 0; q < NB; ++q) {
        const int v = threadIdx.x + 256 * q, row = v >> 3, mm = (v & 7) * 4;
        pb[q] = *reinterpret_cast<const float4*>(basis + (int64_t)(tile * kTokTile + row) * r_pad + m0 + mm);
      }
#pragma unroll
      for (int q = 0; q < NC; ++q) {
        const int v = threadIdx.x + 256 * q, mm = v / (D / 4), c4 = (v % (D / 4)) * 4;
        float4 s4 = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int s = 0; s < splits; ++s) {   // fixed order over the token splits
          const float4 p = *reinterpret_cast<const float4*>(cf + ((int64_t)s * r_pad + m0 + mm) * D + c4);
          s4.x += p.x; s4.y += p.y; s4.z += p.z; s4.w += p.w;
        }
        pc[q] = s4;
      }
    };
    fetch(0);
    for (int m0 = 0; m0 < r_pad; m0 += 32) {
      if (m0 == re_pad) {                   // the even modes are done: park E, start O
#pragma unroll
        for (int j = 0; j < TPW; ++j) {
          acc_e[j] = acc[j];
#pragma unroll
          for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
        }
      }
#pragma unroll
      for (int q = 0; q < NB; ++q) {
        const int v = threadIdx.x + 256 * q, row = v >> 3, mm = (v & 7) * 4;
        Bs[row][mm] = pb[q].x; Bs[row][mm + 1] = pb[q].y; Bs[row][mm + 2] = pb[q].z; Bs[row][mm + 3] = pb[q].w;
      }
#pragma unroll
      for (int q = 0; q < NC; ++q) {
        const int v = threadIdx.x + 256 * q, mm = v / (D / 4), c4 = (v % (D / 4)) * 4;
        *reinterpret_cast<float4*>(&Cs[mm][c4]) = pc[q];
      }
      __syncthreads();
      if (m0 + 32 < r_pad) fetch(m0 + 32);
      // operands of step k+1 are read from LDS while the matrix cores work on step k
      float a_op[2], b_op[2][TPW];
      a_op[0] = Bs[tb * 32 + l32][lhi];
#pragma unroll
      for (int j = 0; j < TPW; ++j) b_op[0][j] = Cs[lhi][cw * (D / 2) + j * 32 + l32];
#pragma unroll
      for (int kk = 0; kk < 16; ++kk) {
        const int cur = kk & 1, nxt = cur ^ 1;
        if (kk + 1 < 16) {
          a_op[nxt] = Bs[tb * 32 + l32][2 * (kk + 1) + lhi];
#pragma unroll
          for (int j = 0; j < TPW; ++j) b_op[nxt][j] = Cs[2 * (kk + 1) + lhi][cw * (D / 2) + j * 32 + l32];
        }
        __builtin_amdgcn_sched_barrier(0);  // keep the reads ahead of the products they overlap with
#pragma unroll
        for (int j = 0; j < TPW; ++j)
          acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_op[cur], b_op[cur][j], acc[j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
      __syncthreads();
    }

    if (re_pad == r_pad) {                  // r = 1: no odd modes
#pragma unroll
      for (int j = 0; j < TPW; ++j) acc_e[j] = acc[j];
    } else {
#pragma unroll
      for (int j = 0; j < TPW; ++j) acc_o[j] = acc[j];
    }
    // epilogue: residuals of tokens i and N-1-i against the stored input, squared, summed over
    // this wave's columns
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      int row = tb * 32 + 8 * (i >> 2) + 4 * lhi + (i & 3);
      int t0 = tile * kTokTile + row;
      asm volatile("" : "+v"(t0));         // keeps the row addresses from being hoisted above the product loop
      const int t = min(t0, nh - 1), tm = n - 1 - t;       // clamped: rows past nh are masked below
      const float w = t0 < nh ? 1.f : 0.f, wm = (t0 < nh && tm != t) ? 1.f : 0.f;
      float hp = 0.f, tot = 0.f, hpm = 0.f, totm = 0.f;
#pragma unroll
      for (int j = 0; j < TPW; ++j) {
        const int col = cw * (D / 2) + j * 32 + l32;
        const bool inside = col < d;
        const float xv = inside ? w * load_elem<T>(x + (int64_t)t * st.sn + col) : 0.f;
        const float xm = inside ? wm * load_elem<T>(x + (int64_t)tm * st.sn + col) : 0.f;
        const float df = xv - w * (acc_e[j][i] + acc_o[j][i]);
        const float dm = xm - wm * (acc_e[j][i] - acc_o[j][i]);
        hp = fmaf(df, df, hp);
        tot = fmaf(xv, xv, tot);
        hpm = fmaf(dm, dm, hpm);
        totm = fmaf(xm, xm, totm);
      }
#pragma unroll
      for (int off = 16; off >= 1; off >>= 1) {
        hp += __shfl_xor(hp, off, 64);
        tot += __shfl_xor(tot, off, 64);
        hpm += __shfl_xor(hpm, off, 64);
        totm += __shfl_xor(totm, off, 64);
      }
      if (l32 == 0) {
        red[tensor][0][cw][row] = hp;
        red[tensor][1][cw][row] = tot;
        red[tensor][2][cw][row] = hpm;
        red[tensor][3][cw][row] = totm;
      }
      __builtin_amdgcn_sched_barrier(0);    // one row at a time: keeps the loads of later rows from piling up
    }
    __syncthreads();
  }

  if (threadIdx.x < kTokTile) {
    int row = threadIdx.x, t = tile * kTokTile + row, tm = n - 1 - t;
    float hpk = red[0][0][0][row] + red[0][0][1][row];
    float hpv = red[1][0][0][row] + red[1][0][1][row];
    float tk = red[0][1][0][row] + red[0][1][1][row];
    float tv = red[1][1][0][row] + red[1][1][1][row];
    float hpkm = red[0][2][0][row] + red[0][2][1][row];
    float hpvm = red[1][2][0][row] + red[1][2][1][row];
    float tkm = red[0][3][0][row] + red[0][3][1][row];
    float tvm = red[1][3][0][row] + red[1][3][1][row];
    if (t < nh) {
      const int64_t ou = out_unit(um, unit);
      scores[ou * n + t] = hpk / (float)d + hpv / (float)d;
      if (tm != t) scores[ou * n + tm] = hpkm / (float)d + hpvm / (float)d;
    }
    // rows past nh, and the mirror of the middle token, hold zeros
    double e[4] = {(double)hpk + (double)hpkm, (double)hpv + (double)hpvm, (double)tk + (double)tkm,
                   (double)tv + (double)tvm};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) e[q] += __shfl_xor(e[q], off, 64);
    }
    if (row == 0) {
      double* o = epart + ((int64_t)unit * tiles + tile) * 4;
      o[0] = e[0]; o[1] = e[1]; o[2] = e[2]; o[3] = e[3];
    }
  }
}

}  // namespace

// ------------------------------------------------------------------ per-unit energy reduction
// One workgroup per unit sums the per-tile partials in a fixed order (strided then tree).
__global__ __launch_bounds__(256) void energy_reduce_kernel(const double* __restrict__ epart, int tiles,
                                                           double* __restrict__ energy, UnitMap um) {
  __shared__ double sm[4][256];
  const int unit = blockIdx.x;
  double e[4] = {0.0, 0.0, 0.0, 0.0};
  for (int t = threadIdx.x; t < tiles; t += 256) {
    const double* p = epart + ((int64_t)unit * tiles + t) * 4;
    e[0] += p[0]; e[1] += p[1]; e[2] += p[2]; e[3] += p[3];
  }
  for (int q = 0; q < 4; ++q) sm[q][threadIdx.x] = e[q];
  __syncthreads();
  for (int s = 128; s >= 1; s >>= 1) {
    if (threadIdx.x < s)
      for (int q = 0; q < 4; ++q) sm[q][threadIdx.x] += sm[q][threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x < 4) energy[out_unit(um, unit) * 4 + threadIdx.x] = sm[threadIdx.x][0];
}

hipError_t energy_reduce_launch(const double* epart, int tiles, int units, double* energy, UnitMap um,
                                hipStream_t s) {
  ProfileScope ps("energy_reduce_kernel", s);
  hipLaunchKernelGGL(energy_reduce_kernel, dim3(units), dim3(256), 0, s, epart, tiles, energy, um);
  return hipGetLastError();
}

// lowpass[ut] = sum over the retained coefficients C[m][c]^2 of tensor ut (Eq. 11 as written)
__global__ __launch_bounds__(256) void dense_lowpass_kernel(const float* __restrict__ coeff, int splits,
                                                           int r_pad, int d, double* __restrict__ lowpass) {
  __shared__ double sm[256];
  const int ut = blockIdx.x;
  const float* cf = coeff + (size_t)ut * splits * r_pad * d;
  double acc = 0.0;
  for (int i = threadIdx.x; i < r_pad * d; i += 256) {
    float v = 0.f;
    for (int s = 0; s < splits; ++s) v += cf[(size_t)s * r_pad * d + i];
    acc += (double)v * (double)v;
  }
  sm[threadIdx.x] = acc;
  __syncthreads();
  for (int s = 128; s >= 1; s >>= 1) {
    if (threadIdx.x < s) sm[threadIdx.x] += sm[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) lowpass[ut] = sm[0];
}

hipError_t dense_lowpass(const fc_kv_desc& d, const DenseLayout& lay, void* ws, double* lowpass, hipStream_t s) {
  const int n_ut = d.batch * d.layers * d.kv_heads * 2;
  ProfileScope ps("dense_lowpass_kernel", s);
  hipLaunchKernelGGL(dense_lowpass_kernel, dim3(n_ut), dim3(256), 0, s,
                     reinterpret_cast<const float*>(static_cast<char*>(ws) + lay.coeff), lay.splits, lay.r_pad,
                     (d.head_dim + 63) / 64 * 64, lowpass);
  return hipGetLastError();
}

// ------------------------------------------------------------------ host side
DenseLayout dense_layout(const fc_kv_desc& d, int32_t r) {
  DenseLayout lay{};
  const int64_t units = (int64_t)d.batch * d.layers * d.kv_heads;
  const int nh = (d.n_tokens + 1) / 2;               // folded rows
  const int re = (r + 1) / 2, ro = r / 2;            // even / odd modes below r
  lay.re_pad = (re + kMTile - 1) / kMTile * kMTile;
  lay.r_pad = lay.re_pad + (ro + kMTile - 1) / kMTile * kMTile;
  lay.n_pad = (nh + kTokTile - 1) / kTokTile * kTokTile;
  lay.tiles = lay.n_pad / kTokTile;
  const int64_t wgs = (int64_t)(lay.r_pad / kMTile) * units * 2;
  int splits = 1;
  if (wgs < 1024) {
    int64_t want = (1024 + wgs - 1) / (wgs > 0 ? wgs : 1);
    int64_t max_splits = lay.n_pad / 256 > 0 ? lay.n_pad / 256 : 1;
    splits = (int)(want < max_splits ? want : max_splits);
  }
  lay.tok_per_split = ((lay.n_pad + splits - 1) / splits + kTokChunk - 1) / kTokChunk * kTokChunk;
  lay.splits = (lay.n_pad + lay.tok_per_split - 1) / lay.tok_per_split;
  auto up = [](size_t x) { return (x + kWsAlign - 1) / kWsAlign * kWsAlign; };
  size_t off = sizeof(WsHeader);
  lay.basis = off; off = up(off + (size_t)lay.n_pad * lay.r_pad * sizeof(float));
  const size_t d_pad = (size_t)(d.head_dim + 63) / 64 * 64;   // the kernels work on head dims padded to 64
  lay.coeff = off; off = up(off + (size_t)units * 2 * lay.splits * lay.r_pad * d_pad * sizeof(float));
  lay.epart = off; off = up(off + (size_t)units * lay.tiles * 4 * sizeof(double));
  lay.total = off;
  return lay;
}

hipError_t dense_prepare(const fc_kv_desc& d, int32_t r, const DenseLayout& lay, void* ws, hipStream_t s) {
  char* base = static_cast<char*>(ws);
  int64_t total = (int64_t)lay.n_pad * lay.r_pad;
  dim3 grid((unsigned)((total + 255) / 256));
  hipLaunchKernelGGL(dense_basis_kernel, grid, dim3(256), 0, s, reinterpret_cast<WsHeader*>(base),
                     reinterpret_cast<float*>(base + lay.basis), d.n_tokens, r, lay.re_pad, lay.r_pad,
                     lay.n_pad, d.head_dim, d.dtype);
  return hipGetLastError();
}

template <typename T, int TPW>
static hipError_t dense_score_t(const void* K, const void* V, const fc_kv_desc& d, int32_t r,
                                const DenseLayout& lay, float* scores, double* energy, void* ws,
                                UnitMap um, hipStream_t s) {
  char* base = static_cast<char*>(ws);
  WsHeader* hdr = reinterpret_cast<WsHeader*>(base);
  float* basis = reinterpret_cast<float*>(base + lay.basis);
  float* coeff = reinterpret_cast<float*>(base + lay.coeff);
  double* epart = reinterpret_cast<double*>(base + lay.epart);
  const int units = d.batch * d.layers * d.kv_heads;
  KvStrides st = strides_of(d);
  dim3 g1(lay.r_pad / kMTile, lay.splits, units * 2);
  {
  ProfileScope ps("dense_coeff_kernel", s);
  hipLaunchKernelGGL((dense_coeff_kernel<T, TPW>), g1, dim3(256), 0, s, static_cast<const T*>(K),
                     static_cast<const T*>(V), st, d.n_tokens, r, lay.re_pad, lay.r_pad, lay.n_pad,
                     lay.tok_per_split, lay.splits, hdr, basis, coeff, d.dtype, d.head_dim);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  dim3 g2(lay.tiles, units);
  {
  ProfileScope ps("dense_score_kernel", s);
  hipLaunchKernelGGL((dense_score_kernel<T, TPW>), g2, dim3(256), 0, s, static_cast<const T*>(K),
                     static_cast<const T*>(V), st, d.n_tokens, r, lay.re_pad, lay.r_pad, lay.splits, hdr,
                     basis, coeff, scores, epart, lay.tiles, d.dtype, d.head_dim, um);
  }
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  return energy_reduce_launch(epart, lay.tiles, units, energy, um, s);
}

hipError_t dense_score(const void* K, const void* V, const fc_kv_desc& d, int32_t r,
                       const DenseLayout& lay, float* scores, double* energy, void* ws, UnitMap um,
                       hipStream_t s) {
  const int tpw = (d.head_dim + 63) / 64;
#define FC_DENSE_CASE(TP)                                                                         \
  case TP:                                                                                        \
    return d.dtype == FC_BF16                                                                     \
               ? dense_score_t<uint16_t, TP>(K, V, d, r, lay, scores, energy, ws, um, s)          \
               : dense_score_t<float, TP>(K, V, d, r, lay, scores, energy, ws, um, s);
  switch (tpw) {
    FC_DENSE_CASE(1)
    FC_DENSE_CASE(2)
    FC_DENSE_CASE(3)
    FC_DENSE_CASE(4)
    default: return hipErrorInvalidValue;
  }
#undef FC_DENSE_CASE
}

}  // namespace fc
