// Dynamic Budget Allocation Module: per-layer outlier-energy ratio (Eq. 12) and the integer
// quotas handed out under the global budget (paragraph after Eq. 12).
//
// The work is a few hundred flops per sequence; the kernel exists so that budgets are produced on
// the device, in stream order, without a host round trip.  One workgroup per sequence: the ratios,
// the shares and the ranking of the fractional parts run one layer per thread; only the sums whose
// rounding order is part of the definition run serially in thread 0.  Everything is IEEE double
// with contraction off, evaluated in exactly the order the header documents, so the result does
// not depend on how the work is spread.
#include "fc_common.h"

namespace fc {

constexpr int kMaxLayers = 1024;
constexpr int kAllocThreads = 256;

#pragma clang fp contract(off)
__global__ __launch_bounds__(kAllocThreads) void allocate_kernel(
    const double* __restrict__ energy, int L, int H, long long T, int b_min, int b_max,
    int* __restrict__ budgets, long long* __restrict__ layer_offsets) {
  __shared__ double R[kMaxLayers];
  __shared__ double q[kMaxLayers];    // share, later its fractional part
  __shared__ double term[kMaxLayers]; // clamp(q) - q of the free layers
  __shared__ int state[kMaxLayers];   // 0 = free, 1 = pinned, 2 = served in the current extra-row round
  __shared__ int bud[kMaxLayers];
  __shared__ double sh_S;
  __shared__ long long sh_left, sh_tleft;
  __shared__ int sh_fast, sh_nfree, sh_mode;     // sh_mode: what every thread does next (see below)
  const int b = blockIdx.x, tid = threadIdx.x;
  const double* e = energy + (size_t)b * L * H * 4;

  // Eq. 12: head energies are summed (ascending h) before each ratio is formed
  for (int l = tid; l < L; l += kAllocThreads) {
    double hp_k = 0.0, hp_v = 0.0, tot_k = 0.0, tot_v = 0.0;
    for (int h = 0; h < H; ++h) {
      const double* p = e + ((size_t)l * H + h) * 4;
      hp_k += p[0]; hp_v += p[1]; tot_k += p[2]; tot_v += p[3];
    }
    const double rk = tot_k > 0.0 ? hp_k / tot_k : 0.0;
    const double rv = tot_v > 0.0 ? hp_v / tot_v : 0.0;
    R[l] = rk + rv;
    state[l] = 0;
    bud[l] = 0;
  }
  __syncthreads();

  if (tid == 0) {
    bool bad = false;
    double s_all = 0.0;
    for (int l = 0; l < L; ++l) {
      const double r = R[l];
      s_all += r;
      if (!isfinite(r) || r < 0.0) bad = true;
    }
    sh_mode = (bad || !isfinite(s_all) || s_all <= 0.0) ? 1 : 0;
    sh_tleft = T;
    sh_nfree = L;
  }
  __syncthreads();
  if (sh_mode == 1)
    for (int l = tid; l < L; l += kAllocThreads) R[l] = 1.0;
  __syncthreads();

  // Share / clamp rounds.  The sums run serially in thread 0, in ascending layer order (their
  // rounding is part of the definition); the divisions, clamps and pins run one layer per thread.
  const double lo = (double)b_min, hi = (double)b_max;
  while (true) {
    if (tid == 0) {
      int mode = 0;                          // 0: shares follow; 2: only zero ratios left; 3: nothing free
      if (sh_nfree <= 0) mode = 3;
      else {
        double S = 0.0;
        for (int l = 0; l < L; ++l)
          if (!state[l]) S += R[l];
        sh_S = S;
        if (S <= 0.0) mode = 2;              // only zero-ratio layers are left: share evenly
      }
      sh_mode = mode;
    }
    __syncthreads();
    const int mode = sh_mode;
    if (mode == 3) break;
    if (mode == 2) {
      for (int l = tid; l < L; l += kAllocThreads)
        if (!state[l]) R[l] = 1.0;
      __syncthreads();
      continue;
    }
    const double S = sh_S;
    const long long t_left = sh_tleft;
    int out = 0;                             // bit 0: some share below b_min, bit 1: some above b_max
    for (int l = tid; l < L; l += kAllocThreads) {
      if (state[l]) continue;
      const double ql = ((double)t_left * R[l]) / S;
      q[l] = ql;
      const double clamped = ql < lo ? lo : (ql > hi ? hi : ql);
      term[l] = clamped - ql;
      out |= (ql < lo ? 1 : 0) | (ql > hi ? 2 : 0);
    }
    if (!__syncthreads_or(out)) break;       // every share is inside the bounds
    if (tid == 0) {
      double viol = 0.0;
      for (int l = 0; l < L; ++l)
        if (!state[l]) viol += term[l];
      const bool pin_under = viol >= 0.0, pin_over = viol <= 0.0;
      long long tl = sh_tleft;
      int nf = sh_nfree;
      for (int l = 0; l < L; ++l) {
        if (state[l]) continue;
        if (pin_under && q[l] < lo) { bud[l] = b_min; tl -= b_min; state[l] = 1; --nf; }
        else if (pin_over && q[l] > hi) { bud[l] = b_max; tl -= b_max; state[l] = 1; --nf; }
      }
      sh_tleft = tl;
      sh_nfree = nf;
    }
    __syncthreads();
  }

  if (tid == 0) {
    const long long t_left = sh_tleft;
    const int n_free = sh_nfree;
    long long left = 0;
    int fast = 1;
    if (n_free == 1) {
      for (int l = 0; l < L; ++l)
        if (!state[l]) bud[l] = (int)t_left;
    } else if (n_free > 1) {
      long long sum_floor = 0;
      for (int l = 0; l < L; ++l) {
        if (state[l]) continue;
        const double f = floor(q[l]);
        bud[l] = (int)f;
        q[l] = q[l] - f;                   // q now holds the fractional part
        sum_floor += (long long)f;
        if (bud[l] >= b_max) fast = 0;     // an extra row could break the bound: take the slow route
      }
      left = t_left - sum_floor;
      if (left < 0 || left >= n_free) fast = 0;
    }
    sh_left = left;
    sh_fast = fast;
  }
  __syncthreads();

  const long long left = sh_left;
  if (sh_fast) {
    // the `left` largest fractional parts (ties to the lower layer) get one more row each:
    // layer l is served iff fewer than `left` free layers rank before it
    for (int l = tid; l < L; l += kAllocThreads) {
      if (state[l] || left <= 0) continue;
      const double fl = q[l];
      int before = 0;
      for (int m = 0; m < L; ++m)
        if (!state[m] && (q[m] > fl || (q[m] == fl && m < l))) ++before;
      if (before < left) bud[l] += 1;
    }
  } else if (tid == 0) {
    // rare: rounding left an unusual number of rows over, or a layer sits at its upper bound.
    // Serve layers in the same order, skipping those at a bound, in as many rounds as needed.
    long long rem = left;
    while (rem > 0) {
      int best = -1;
      for (int l = 0; l < L; ++l)
        if (state[l] == 0 && bud[l] < b_max && (best < 0 || q[l] > q[best])) best = l;
      if (best < 0) {
        bool any = false;
        for (int l = 0; l < L; ++l)
          if (state[l] == 2) { state[l] = 0; any |= bud[l] < b_max; }
        if (!any) break;
        continue;
      }
      bud[best] += 1; state[best] = 2; --rem;
    }
    while (rem < 0) {
      int best = -1;
      for (int l = L - 1; l >= 0; --l)
        if (state[l] == 0 && bud[l] > b_min && (best < 0 || q[l] < q[best])) best = l;
      if (best < 0) {
        bool any = false;
        for (int l = 0; l < L; ++l)
          if (state[l] == 2) { state[l] = 0; any |= bud[l] > b_min; }
        if (!any) break;
        continue;
      }
      bud[best] -= 1; state[best] = 2; ++rem;
    }
  }
  __syncthreads();

  for (int l = tid; l < L; l += kAllocThreads) budgets[(size_t)b * L + l] = bud[l];
  if (tid == 0) {
    long long off = 0;
    long long* offs = layer_offsets + (size_t)b * (L + 1);
    offs[0] = 0;
    for (int l = 0; l < L; ++l) {
      off += (long long)H * bud[l];
      offs[l + 1] = off;
    }
  }
}

hipError_t allocate_launch(const double* energy, int32_t B, int32_t L, int32_t H, int32_t N, int64_t T,
                           int32_t b_min, int32_t b_max, int32_t* budgets, int64_t* layer_offsets,
                           hipStream_t s) {
  (void)N;
  ProfileScope ps("allocate_kernel", s);
  hipLaunchKernelGGL(allocate_kernel, dim3(B), dim3(kAllocThreads), 0, s, energy, L, H, (long long)T, b_min,
                     b_max, budgets, reinterpret_cast<long long*>(layer_offsets));
  return hipGetLastError();
}

}  // namespace fc
