// Selection of the b_l highest-scoring KV pairs of every unit and the packed gather (the rule in
// the sentence after Eq. 10: per layer, the pairs that deviate most, as many as the budget allows).
//
// select_kernel / select_large_kernel: one workgroup per unit.  A four-pass 8-bit radix select
//   over the fp32 bit patterns finds the k-th largest key and how many keys equal to it are
//   still needed; a compaction in token order (prefix counts) then writes the kept indices, which
//   yields them ascending and gives ties to the lower index without any sort.  Up to 65536
//   tokens the keys stay in registers between the passes; beyond that they are re-read from L2.
//   Only integer atomics are used (LDS histogram), so the result is deterministic.
// gather_kernel: one 16-byte vector per thread; rows are bit copies.
#include "fc_common.h"

namespace fc {

namespace {

constexpr int kSelThreads = 1024;

// Monotone map float -> uint32 (larger float = larger key), valid for any sign.
__device__ __forceinline__ uint32_t order_key(float f) {
  uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Score the selection is taken on.  Per-head mode: the unit's own score.  Layer-shared mode (the
// row-wide reading of Eq. 10, where the MSE runs over all H*d features of a token): the fp32 sum
// of the heads' scores in ascending head order divided by H, one correctly rounded division.
template <bool SHARED>
__device__ __forceinline__ float score_at(const float* __restrict__ s, int i, int n, int H) {
  if (!SHARED) return s[i];
  float acc = s[i];
  for (int h = 1; h < H; ++h) acc += s[(size_t)h * n + i];
  return __fdiv_rn(acc, (float)H);
}

template <bool SHARED>
__global__ __launch_bounds__(kSelThreads) void select_large_kernel(
    const float* __restrict__ scores, const int* __restrict__ budgets,
    const long long* __restrict__ layer_offsets, int L, int H, int n, long long rows_per_seq,
    int* __restrict__ idx_out) {
  __shared__ unsigned hist[256];
  __shared__ unsigned wave_gt[kSelThreads / 64], wave_eq[kSelThreads / 64];
  __shared__ unsigned sh_bucket, sh_need;
  __shared__ unsigned run_gt, run_eq;

  // per-head mode: one workgroup per (b,l,h); layer-shared mode: one per (b,l), writing H copies
  const int unit = SHARED ? blockIdx.x * H : blockIdx.x;
  const int h = unit % H, bl = unit / H, l = bl % L, b = bl / L;
  const int k = budgets[(size_t)b * L + l];
  const int copies = SHARED ? H : 1;
  const long long off = layer_offsets[(size_t)b * (L + 1) + l] + (long long)h * k;
  if (k <= 0 || k > n || off < 0 || off + (long long)copies * k > rows_per_seq) return;   // bad budgets
  const float* s = scores + (size_t)unit * n;
  int* out = idx_out + (size_t)b * rows_per_seq + off;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  // ---- radix select: after the loop `prefix` is the k-th largest key
  uint32_t prefix = 0, mask = 0;
  unsigned need = (unsigned)k;
  for (int shift = 24; shift >= 0; shift -= 8) {
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    for (int i = tid; i < n; i += kSelThreads) {
      uint32_t key = order_key(score_at<SHARED>(s, i, n, H));
      if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
    }
    __syncthreads();
    if (wave == 0) {
      // suffix sums over the 256 buckets, 4 per lane (lane 63 holds the top buckets)
      unsigned c0 = hist[lane * 4 + 0], c1 = hist[lane * 4 + 1], c2 = hist[lane * 4 + 2],
               c3 = hist[lane * 4 + 3];
      unsigned mine = c0 + c1 + c2 + c3;
      unsigned above = 0;                      // keys in buckets of higher lanes
      unsigned run = mine;
#pragma unroll
      for (int d = 1; d < 64; d <<= 1) {
        unsigned v = __shfl_down(run, d, 64);
        if (lane + d < 64) run += v;
      }
      above = run - mine;
      // the bucket holding the need-th largest key is in this lane iff above < need <= above+mine
      if (above < need && need <= above + mine) {
        unsigned a = above;
        unsigned bucket;
        if (a + c3 >= need) bucket = 3;
        else { a += c3; if (a + c2 >= need) bucket = 2;
        else { a += c2; if (a + c1 >= need) bucket = 1;
        else { a += c1; bucket = 0; } } }
        sh_bucket = lane * 4 + bucket;
        sh_need = need - a;
      }
    }
    __syncthreads();
    prefix |= sh_bucket << shift;
    mask |= 255u << shift;
    need = sh_need;
    __syncthreads();
  }
  const uint32_t tau = prefix;          // key of the k-th largest score
  // `need` = how many keys equal to tau are kept (those with the lowest token indices)

  // ---- compaction in token order
  if (tid == 0) { run_gt = 0; run_eq = 0; }
  __syncthreads();
  for (int base = 0; base < n; base += kSelThreads) {
    const int i = base + tid;
    uint32_t key = i < n ? order_key(score_at<SHARED>(s, i, n, H)) : 0u;
    const bool gt = i < n && key > tau;
    const bool eq = i < n && key == tau;
    const unsigned long long bgt = __ballot(gt), beq = __ballot(eq);
    const unsigned long long below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    const unsigned pre_gt = __popcll(bgt & below), pre_eq = __popcll(beq & below);
    if (lane == 0) { wave_gt[wave] = __popcll(bgt); wave_eq[wave] = __popcll(beq); }
    __syncthreads();
    unsigned ogt = run_gt, oeq = run_eq, tgt = 0, teq = 0;
#pragma unroll
    for (int w = 0; w < kSelThreads / 64; ++w) {
      unsigned g = wave_gt[w], e = wave_eq[w];
      if (w < wave) { ogt += g; oeq += e; }
      tgt += g; teq += e;
    }
    const unsigned gt_before = ogt + pre_gt, eq_before = oeq + pre_eq;
    if (gt || (eq && eq_before < need)) {
      const unsigned pos = gt_before + min(eq_before, need);
      for (int c = 0; c < copies; ++c) out[(size_t)c * k + pos] = i;
    }
    __syncthreads();
    if (tid == 0) { run_gt += tgt; run_eq += teq; }
    __syncthreads();
  }
}

// Register-resident variant for n <= 64*1024: thread t keeps tokens [t*chunk, (t+1)*chunk) in
// registers (at most MAXC = 32 or 64 of them), so the scores are read once; the ordered compaction
// is one block-wide scan of the per-thread counts followed by sequential writes.
constexpr int kSelMaxChunk = 64;

__device__ __forceinline__ unsigned wave_excl_scan(unsigned v, unsigned& total) {
  const int lane = threadIdx.x & 63;
  unsigned incl = v;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    unsigned o = __shfl_up(incl, d, 64);
    if (lane >= d) incl += o;
  }
  total = __shfl(incl, 63, 64);
  return incl - v;
}

template <bool SHARED, int MAXC>
__global__ __launch_bounds__(kSelThreads) void select_kernel(
    const float* __restrict__ scores, const int* __restrict__ budgets,
    const long long* __restrict__ layer_offsets, int L, int H, int n, int chunk, long long rows_per_seq,
    int* __restrict__ idx_out) {
  __shared__ unsigned hist[256];
  __shared__ unsigned wave_gt[kSelThreads / 64], wave_eq[kSelThreads / 64];
  __shared__ unsigned sh_bucket, sh_need;

  // per-head mode: one workgroup per (b,l,h); layer-shared mode: one per (b,l), writing H copies
  const int unit = SHARED ? blockIdx.x * H : blockIdx.x;
  const int h = unit % H, bl = unit / H, l = bl % L, b = bl / L;
  const int k = budgets[(size_t)b * L + l];
  const int copies = SHARED ? H : 1;
  const long long off = layer_offsets[(size_t)b * (L + 1) + l] + (long long)h * k;
  if (k <= 0 || k > n || off < 0 || off + (long long)copies * k > rows_per_seq) return;   // bad budgets
  const float* s = scores + (size_t)unit * n;
  int* out = idx_out + (size_t)b * rows_per_seq + off;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int i0 = tid * chunk;

  // keys of this thread's chunk; positions past n get key 0, below every real key (real keys of
  // non-negative floats have the top bit set, of negative floats are >= 1 unless the score is NaN)
  uint32_t key[MAXC];
  if (!SHARED && (chunk & 3) == 0 && (n & 3) == 0 && (reinterpret_cast<uintptr_t>(s) & 15u) == 0) {
#pragma unroll
    for (int j = 0; j < MAXC; j += 4) {
      float4 f = make_float4(0.f, 0.f, 0.f, 0.f);
      const bool in = j < chunk && i0 + j < n;
      if (in) f = *reinterpret_cast<const float4*>(s + i0 + j);
      key[j] = in ? order_key(f.x) : 0u; key[j + 1] = in ? order_key(f.y) : 0u;
      key[j + 2] = in ? order_key(f.z) : 0u; key[j + 3] = in ? order_key(f.w) : 0u;
    }
  } else {
#pragma unroll
    for (int j = 0; j < MAXC; ++j) {
      const bool in = j < chunk && i0 + j < n;
      key[j] = in ? order_key(score_at<SHARED>(s, i0 + j, n, H)) : 0u;
    }
  }
  const int mine = max(0, min(chunk, n - i0));     // valid keys of this thread

  uint32_t prefix = 0, mask = 0;
  unsigned need = (unsigned)k;
  for (int shift = 24; shift >= 0; shift -= 8) {
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    unsigned run_dig = 0, run_cnt = 0;
#pragma unroll
    for (int j = 0; j < MAXC; ++j) {
      // neighbouring keys mostly share their leading digits, so runs of equal digits are counted
      // in a register and flushed with one atomic (integer adds: the histogram is the same)
      const bool in = j < mine && (key[j] & mask) == prefix;
      const unsigned dig = (key[j] >> shift) & 255u;
      if (in && run_cnt > 0 && dig == run_dig) {
        ++run_cnt;
      } else {
        if (run_cnt > 0) atomicAdd(&hist[run_dig], run_cnt);
        run_dig = dig;
        run_cnt = in ? 1u : 0u;
      }
    }
    if (run_cnt > 0) atomicAdd(&hist[run_dig], run_cnt);
    __syncthreads();
    if (wave == 0) {
      unsigned c0 = hist[lane * 4 + 0], c1 = hist[lane * 4 + 1], c2 = hist[lane * 4 + 2],
               c3 = hist[lane * 4 + 3];
      unsigned mine4 = c0 + c1 + c2 + c3;
      unsigned run = mine4;
#pragma unroll
      for (int d = 1; d < 64; d <<= 1) {
        unsigned v = __shfl_down(run, d, 64);
        if (lane + d < 64) run += v;
      }
      const unsigned above = run - mine4;
      if (above < need && need <= above + mine4) {
        unsigned a = above, bucket;
        if (a + c3 >= need) bucket = 3;
        else { a += c3; if (a + c2 >= need) bucket = 2;
        else { a += c2; if (a + c1 >= need) bucket = 1;
        else { a += c1; bucket = 0; } } }
        sh_bucket = lane * 4 + bucket;
        sh_need = need - a;
      }
    }
    __syncthreads();
    prefix |= sh_bucket << shift;
    mask |= 255u << shift;
    need = sh_need;
  }
  const uint32_t tau = prefix;

  unsigned cg = 0, ce = 0;
#pragma unroll
  for (int j = 0; j < MAXC; ++j) {
    cg += (j < mine && key[j] > tau) ? 1u : 0u;
    ce += (j < mine && key[j] == tau) ? 1u : 0u;
  }
  unsigned tg, te;
  unsigned pg = wave_excl_scan(cg, tg), pe = wave_excl_scan(ce, te);
  if (lane == 0) { wave_gt[wave] = tg; wave_eq[wave] = te; }
  __syncthreads();
  for (int w = 0; w < wave; ++w) { pg += wave_gt[w]; pe += wave_eq[w]; }
  // pg / pe = kept-candidates strictly before this thread's chunk (greater / equal to tau)
#pragma unroll
  for (int j = 0; j < MAXC; ++j) {
    if (j < mine) {
      const bool gt = key[j] > tau, eq = key[j] == tau;
      if (gt || (eq && pe < need)) {
        const unsigned pos = pg + min(pe, need);
        for (int c = 0; c < copies; ++c) out[(size_t)c * k + pos] = i0 + j;
      }
      pg += gt ? 1u : 0u;
      pe += eq ? 1u : 0u;
    }
  }
}

// Destination of the paged variant: kept row j of unit (b,l,h) goes to slot j % page_size of page
// block_table[b][l][h][j / page_size] of caches laid out [num_pages][page_size][d].
struct PagedDst {
  const int* block_table;
  int page_size, max_pages;
  long long num_pages;
};

// One thread copies one 16-byte vector of a K row and of the matching V row; blockIdx.y is the
// sequence.  Rows are read once and written once, so both sides bypass the caches' retention
// (non-temporal): the scores, budgets and indices the other lanes need stay resident instead.
typedef unsigned int uint4v __attribute__((ext_vector_type(4)));

template <bool PAGED>
__global__ __launch_bounds__(256) void gather_kernel(
    const char* __restrict__ K, const char* __restrict__ V, KvStrides st, int n, int elem_bytes,
    int vec_per_row, int vpr_shift, const int* __restrict__ budgets,
    const long long* __restrict__ layer_offsets, const int* __restrict__ idx, long long rows_per_seq,
    char* __restrict__ K_out, char* __restrict__ V_out, PagedDst pg) {
  const int b = blockIdx.y;
  const long long v = (long long)blockIdx.x * blockDim.x + threadIdx.x;     // vector within the sequence
  const long long j = vpr_shift >= 0 ? (v >> vpr_shift) : v / vec_per_row;   // packed row of the sequence
  const int part = (int)(vpr_shift >= 0 ? (v & (vec_per_row - 1)) : v % vec_per_row);
  if (j >= rows_per_seq) return;
  const long long* offs = layer_offsets + (size_t)b * (st.L + 1);
  // largest l with offs[l] <= j
  int lo = 0, hi = st.L;                                // invariant: offs[lo] <= j < offs[hi]
  if (j >= offs[st.L]) return;                          // rows beyond what the budgets fill
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (offs[mid] <= j) lo = mid; else hi = mid;
  }
  const int l = lo;
  const int k = budgets[(size_t)b * st.L + l];
  if (k <= 0) return;
  const long long in_layer = j - offs[l];                // < H * k
  if (in_layer >= (long long)st.H * k) return;
  const int h = (int)((unsigned)in_layer / (unsigned)k);
  const long long grow = (long long)b * rows_per_seq + j;
  const int token = idx[grow];
  if (token < 0 || token >= n) return;
  const long long src = ((long long)b * st.sb + (long long)l * st.sl + (long long)h * st.sh +
                         (long long)token * st.sn) * elem_bytes + (long long)part * 16;
  long long dst_row = grow;
  if (PAGED) {
    const long long jj = in_layer - (long long)h * k;                // row within the unit
    const long long slot_page = jj / pg.page_size;
    if (slot_page >= pg.max_pages) return;
    const long long unit = ((long long)b * st.L + l) * st.H + h;
    const long long page = pg.block_table[unit * pg.max_pages + slot_page];
    if (page < 0 || page >= pg.num_pages) return;                    // not a valid page: row skipped
    dst_row = page * pg.page_size + jj % pg.page_size;
  }
  const long long dst = dst_row * (long long)vec_per_row * 16 + (long long)part * 16;
  const uint4v kv = __builtin_nontemporal_load(reinterpret_cast<const uint4v*>(K + src));
  const uint4v vv = __builtin_nontemporal_load(reinterpret_cast<const uint4v*>(V + src));
  __builtin_nontemporal_store(kv, reinterpret_cast<uint4v*>(K_out + dst));
  __builtin_nontemporal_store(vv, reinterpret_cast<uint4v*>(V_out + dst));
}

}  // namespace

hipError_t select_gather_launch(const void* K, const void* V, const fc_kv_desc& d, const float* scores,
                                const int32_t* budgets, const int64_t* layer_offsets,
                                int64_t rows_per_seq, bool shared, int32_t* idx_out, void* K_out,
                                void* V_out, const int32_t* block_table, int32_t page_size,
                                int32_t max_pages, int64_t num_pages, hipStream_t s) {
  const int units = d.batch * d.layers * d.kv_heads;
  if (units == 0 || rows_per_seq == 0) return hipSuccess;
  const long long* offs = reinterpret_cast<const long long*>(layer_offsets);
  {
    ProfileScope ps(shared ? "select_shared_kernel" : "select_kernel", s);
    const int chunk = (d.n_tokens + kSelThreads - 1) / kSelThreads;
    const dim3 grid(shared ? units / d.kv_heads : units), block(kSelThreads);
    const long long rows = (long long)rows_per_seq;
    if (chunk <= 32) {
      if (shared)
        hipLaunchKernelGGL((select_kernel<true, 32>), grid, block, 0, s, scores, budgets, offs, d.layers,
                           d.kv_heads, d.n_tokens, (chunk + 3) & ~3, rows, idx_out);
      else
        hipLaunchKernelGGL((select_kernel<false, 32>), grid, block, 0, s, scores, budgets, offs, d.layers,
                           d.kv_heads, d.n_tokens, (chunk + 3) & ~3, rows, idx_out);
    } else if (chunk <= kSelMaxChunk && !shared) {   // (the layer-shared keys need too many registers)
      hipLaunchKernelGGL((select_kernel<false, 64>), grid, block, 0, s, scores, budgets, offs, d.layers,
                         d.kv_heads, d.n_tokens, (chunk + 3) & ~3, rows, idx_out);
    } else {
      if (shared)
        hipLaunchKernelGGL(select_large_kernel<true>, grid, block, 0, s, scores, budgets, offs, d.layers,
                           d.kv_heads, d.n_tokens, rows, idx_out);
      else
        hipLaunchKernelGGL(select_large_kernel<false>, grid, block, 0, s, scores, budgets, offs, d.layers,
                           d.kv_heads, d.n_tokens, rows, idx_out);
    }
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int elem_bytes = d.dtype == FC_BF16 ? 2 : 4;
  const int vec_per_row = d.head_dim * elem_bytes / 16;
  const long long seq_vecs = (long long)rows_per_seq * vec_per_row;
  const long long blocks = (seq_vecs + 255) / 256;
  if (blocks > 0x7FFFFFFFll || d.batch > 65535) return hipErrorInvalidValue;
  int vpr_shift = -1;
  if ((vec_per_row & (vec_per_row - 1)) == 0)
    for (vpr_shift = 0; (1 << vpr_shift) < vec_per_row; ++vpr_shift) {}
  ProfileScope ps("gather_kernel", s);
  const PagedDst pg{block_table, page_size, max_pages, (long long)num_pages};
  const dim3 grid((unsigned)blocks, (unsigned)d.batch);
  if (block_table)
    hipLaunchKernelGGL(gather_kernel<true>, grid, dim3(256), 0, s, static_cast<const char*>(K),
                       static_cast<const char*>(V), strides_of(d), d.n_tokens, elem_bytes, vec_per_row,
                       vpr_shift, budgets, offs, idx_out, (long long)rows_per_seq, static_cast<char*>(K_out),
                       static_cast<char*>(V_out), pg);
  else
    hipLaunchKernelGGL(gather_kernel<false>, grid, dim3(256), 0, s, static_cast<const char*>(K),
                       static_cast<const char*>(V), strides_of(d), d.n_tokens, elem_bytes, vec_per_row,
                       vpr_shift, budgets, offs, idx_out, (long long)rows_per_seq, static_cast<char*>(K_out),
                       static_cast<char*>(V_out), pg);
  return hipGetLastError();
}

}  // namespace fc
