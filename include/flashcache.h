/*
 * flashcache.h - C ABI of the prefill-time KV-cache compression hot path for MI355X (gfx950).
 *
 * The path is the one-shot compression applied to the KV cache after prefill
 * (Method section, "FlashCache"): the Outlier KV Recognition Module (Eq. 5-10)
 * scores every KV pair by its deviation from the low-pass "Base KV", the Dynamic
 * Budget Allocation Module (Eq. 11-12 and the paragraph after them) turns the
 * per-layer share of high-frequency energy into per-layer quotas, and the
 * highest-scoring pairs of every layer are kept and compacted.
 *
 * Conventions shared by every entry point
 *   - Plain C types only.  Every pointer named "device" is caller-owned device
 *     memory; "host" pointers are ordinary host memory.  The library allocates
 *     and frees nothing; scratch space comes in through `workspace`.
 *   - All work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL =
 *     the default stream) and the call returns without synchronising.  Calls on
 *     one stream execute in order, so score -> allocate -> select_gather needs no
 *     host synchronisation in between: budgets are consumed on the device.
 *   - Shapes and pointers are validated on the host before anything is launched;
 *     on any error nothing is enqueued and a status code is returned (nothing is
 *     printed, no exception crosses the boundary).
 *   - Inputs must be finite.  NaN/Inf give unspecified scores (never a fault).
 *   - Outputs are bit-identical for identical inputs (no floating-point atomics).
 *
 * Notation: B sequences, L layers, H KV heads, N tokens, d head dim, one "unit"
 * is one (sequence, layer, head).  T is the global budget in rows per head summed
 * over the layers of one sequence; every head of layer l keeps b_l rows and
 * sum_l b_l = T, so the packed output of a sequence always has exactly H*T rows.
 */
#ifndef FLASHCACHE_H_
#define FLASHCACHE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  FC_OK = 0,
  FC_EINVAL = 1,       /* null pointer, bad shape/stride/alignment, r outside [1, N] */
  FC_EUNSUPPORTED = 2, /* valid request that no kernel in this build covers */
  FC_EWORKSPACE = 3,   /* workspace pointer null/misaligned or too small */
  FC_EBUDGET = 4,      /* L*b_min > T, L*b_max < T, or bounds outside [1, N] */
  FC_EHIP = 5          /* a HIP call or kernel launch failed (hipGetLastError is left set) */
} fc_status;

typedef enum { FC_F32 = 0, FC_BF16 = 1 } fc_dtype;

/* Realisation of the low-pass projection (both compute the same Base KV). */
typedef enum {
  FC_PATH_AUTO = 0,  /* FC_PATH_FFT where it applies, else FC_PATH_DENSE */
  FC_PATH_DENSE = 1, /* explicit basis: C = B^T X, base = B C, on the matrix cores; any N,
                        head_dim <= 256 */
  FC_PATH_FFT = 2    /* fast cosine transform on the vector ALUs: N a multiple of 1024 (up to
                        132 * 1024), or of 256 (up to 64 * 1024, head_dim a multiple of 16);
                        head_dim a multiple of 8; any cut-off 1 <= r <= N */
} fc_path;

/* Layout of K and of V (one descriptor serves both): element (b,l,h,n,c) lives at
 * base + b*stride_b + l*stride_l + h*stride_h + n*stride_n + c, strides in elements,
 * the head dimension contiguous.  Row starts must be 16-byte aligned. */
typedef struct {
  int32_t batch, layers, kv_heads, n_tokens, head_dim; /* B, L, H, N, d */
  int32_t dtype;                                       /* fc_dtype */
  int64_t stride_b, stride_l, stride_h, stride_n;
} fc_kv_desc;

/* ---- host helpers: the only place where the paper's real-valued hyper-parameters
 * become integers --------------------------------------------------------------- */

/* Number r of retained DCT modes for cut-off factor gamma (Eq. 8: modes 0..omega with
 * omega = gamma*N are kept): min(N, floor(gamma*N)+1), at least 1.  Returns 0 if N < 1. */
int32_t flashcache_cutoff_r(int32_t n_tokens, double gamma);

/* Global budget T for retention ratio rho ("a given overall cache ratio", paragraph after
 * Eq. 12): floor(rho*L*N) clamped to [L, L*N].  Returns 0 if L < 1 or N < 1. */
int64_t flashcache_total_budget(int32_t layers, int32_t n_tokens, double rho);

/* The realisation FC_PATH_AUTO resolves to for this shape (FC_PATH_DENSE or FC_PATH_FFT),
 * or 0 if the shape is invalid or unsupported. */
int32_t flashcache_resolve_path(const fc_kv_desc* desc, int32_t r, int32_t path);

/* Bytes of device workspace flashcache_prepare/flashcache_score need for this shape, cut-off
 * and realisation; 0 if the request is invalid or unsupported. */
size_t flashcache_workspace_bytes(const fc_kv_desc* desc, int32_t r, int32_t path);

/* Bytes of device workspace the flashcache_select_gather* entry points need.  The selection kernels
 * of this build keep their histograms in LDS and registers and need none: this returns 0, and the
 * `workspace` / `workspace_bytes` arguments of those entry points are accepted and ignored (NULL, 0
 * is fine); they are part of the signature so that a build whose selection spans several
 * workgroups per unit can ask for scratch without an ABI change. */
size_t flashcache_select_workspace_bytes(const fc_kv_desc* desc);

/* One-time table construction for (N, r, path): the explicit basis alpha[m]*phi_N(m,i) of
 * Eq. 7 for the dense realisation, or the twiddle tables of the fast transform.  Writes only
 * into `workspace` (device, 256-byte aligned, at least flashcache_workspace_bytes()).  The
 * same workspace, shape, r and path must then be passed to flashcache_score; a workspace that
 * was prepared for something else makes the score kernels write nothing and raise the error
 * flag that flashcache_workspace_error() reports. */
fc_status flashcache_prepare(const fc_kv_desc* desc, int32_t r, int32_t path,
                             void* workspace, size_t workspace_bytes, void* hip_stream);

/* Reads back (synchronising `hip_stream`) the error flag kernels raise when they find a
 * workspace that was not prepared for their arguments.  *flag_out (host) is 0 if all is well. */
fc_status flashcache_workspace_error(const void* workspace, int32_t* flag_out, void* hip_stream);

/* Outlier KV Recognition Module (Eq. 6-10) for every unit.
 *   K, V      device, layout per `desc`, dtype per desc->dtype; read only.
 *   r         retained modes, 1 <= r <= N.
 *   scores    device out, float [B][L][H][N]:  Dev[x] = Dev_k[x] + Dev_v[x], where Dev_k[x] is
 *             the mean over the d features of (K[x] - K_base[x])^2 and K_base is the inverse
 *             DCT of the coefficients of K with modes >= r zeroed (Eq. 8-10); same for V.
 *   energy    device out, double [B][L][H][4] = Ehp_k, Ehp_v, Etot_k, Etot_v: energy removed by
 *             the low-pass (= sum over the zeroed modes of |C[m]|^2 by Parseval, Eq. 11) and
 *             total energy ||X||_F^2, the inputs of Eq. 12.
 * Arithmetic: inputs widened exactly to fp32, fp32 accumulation, energies reduced in fp64
 * in a fixed order. */
fc_status flashcache_score(const void* K, const void* V, const fc_kv_desc* desc, int32_t r,
                           int32_t path, float* scores, double* energy,
                           void* workspace, size_t workspace_bytes, void* hip_stream);

/* The same for ONE layer of every sequence, written into layer `layer` of full-size outputs: K, V
 * and `desc` describe [B][1][H][N][d] (desc->layers must be 1, strides as in the full tensors);
 * `scores` is the full float [B][total_layers][H][N] array and `energy` the full double
 * [B][total_layers][H][4] array.  Lets prefill hand layers over one by one (any order, any stream
 * order that keeps the calls on one workspace sequential); allocation and selection run once
 * after the last layer.  Results are bit-identical to one flashcache_score call over all layers. */
fc_status flashcache_score_layer(const void* K, const void* V, const fc_kv_desc* desc, int32_t layer,
                                 int32_t total_layers, int32_t r, int32_t path, float* scores,
                                 double* energy, void* workspace, size_t workspace_bytes,
                                 void* hip_stream);

/* Spectrum-side cross-check of Eq. 11-12.  flashcache_score derives the energy above the cut-off
 * from the residual (Parseval); this call returns the energy BELOW the cut-off computed from the
 * DCT coefficients themselves, sum over m < r of |C[m]|^2, so that Etot - lowpass can be compared
 * with Ehp.  Valid after flashcache_score on the same workspace with the same desc, r and path,
 * and before the workspace is used again.  (For r > N/2 the fast transform works on the dropped
 * modes; it then sums |C[m]|^2 over m >= r, Eq. 12's numerator as written, and returns the total
 * energy minus that sum.)
 *   lowpass_energy  device out, double [B][L][H][2] = (K, V) */
fc_status flashcache_lowpass_energy(const fc_kv_desc* desc, int32_t r, int32_t path, void* workspace,
                                    size_t workspace_bytes, double* lowpass_energy, void* hip_stream);

/* Dynamic Budget Allocation Module (Eq. 12 and the paragraph after it), per sequence:
 *   R^l = sum_h Ehp_k / sum_h Etot_k + sum_h Ehp_v / sum_h Etot_v   (0 for a zero denominator)
 * then integer quotas proportional to R^l under the global budget:
 *   shares q_l = T'*R^l / S over the free layers; while a share is outside [b_min, b_max]
 *   pin the low ones to b_min if sum(clamp(q)-q) > 0, the high ones to b_max if it is < 0
 *   (both if 0) and re-share the rest; then b_l = floor(q_l) and the left-over rows go one
 *   each to the largest fractional parts, ties to the lower layer.  Negative or non-finite
 *   ratios, or a zero sum, give the uniform split.  IEEE double, no contraction.
 *   energy         device in, double [B][L][H][4] as written by flashcache_score
 *   total_budget   T, with L*b_min <= T <= L*b_max and 1 <= b_min <= b_max <= N
 *   budgets        device out, int32 [B][L], sum over l = T
 *   layer_offsets  device out, int64 [B][L+1]: off[0]=0, off[l+1]=off[l]+H*b_l, off[L]=H*T */
fc_status flashcache_allocate(const double* energy, int32_t batch, int32_t layers,
                              int32_t kv_heads, int32_t n_tokens, int64_t total_budget,
                              int32_t b_min, int32_t b_max, int32_t* budgets,
                              int64_t* layer_offsets, void* hip_stream);

/* Keep the b_l highest-scoring KV pairs of every unit and compact them (the selection rule stated
 * in the sentence after Eq. 10: per layer, the pairs with the largest deviation, as many as the
 * layer's budget allows).
 *   scores         device in, float [B][L][H][N]; compared as fp32 values
 *   budgets        device in, int32 [B][L] (0 <= b_l <= N), layer_offsets device in, [B][L+1],
 *                  both as written by flashcache_allocate; rows_per_seq = H*T is the packed
 *                  row count of one sequence (must equal off[L]; it sizes the outputs)
 *   idx_out        device out, int32 [B][H*T]: kept token indices, ordered by layer, then
 *                  head, then ascending token; among equal scores the lower index is kept
 *   K_out, V_out   device out, [B][H*T][d] in the input dtype: bit copies of the kept rows */
fc_status flashcache_select_gather(const void* K, const void* V, const fc_kv_desc* desc,
                                   const float* scores, const int32_t* budgets,
                                   const int64_t* layer_offsets, int64_t rows_per_seq,
                                   int32_t* idx_out, void* K_out, void* V_out,
                                   void* workspace, size_t workspace_bytes, void* hip_stream);

/* Layer-shared variant of flashcache_select_gather: the reading of Eq. 10 in which the MSE of a
 * token runs over the whole row of the layer's K (and V), all H*d features, so that a layer has
 * ONE score per token and every head keeps the same b_l tokens.  The layer score is the fp32 sum
 * of the heads' scores in ascending head order divided by H (one correctly rounded division);
 * selection, tie rule, output layout and all arguments are as for flashcache_select_gather
 * (idx_out repeats the layer's index list once per head). */
fc_status flashcache_select_gather_shared(const void* K, const void* V, const fc_kv_desc* desc,
                                          const float* scores, const int32_t* budgets,
                                          const int64_t* layer_offsets, int64_t rows_per_seq,
                                          int32_t* idx_out, void* K_out, void* V_out,
                                          void* workspace, size_t workspace_bytes, void* hip_stream);

/* Variant that compacts straight into a paged KV cache instead of a packed buffer (so that the
 * compacted cache can be handed to a paged decode kernel without another copy).  Selection is
 * as in flashcache_select_gather (shared = 0) or flashcache_select_gather_shared (shared != 0);
 * idx_out is written as before.  Kept row j (0 <= j < b_l, ascending token order) of unit (b,l,h)
 * is copied to slot j % page_size of page block_table[b][l][h][j / page_size]:
 *   block_table   device in, int32 [B][L][H][max_pages], the pages of each unit in order
 *   K_cache/V_cache  device out, [num_pages][page_size][d] in the input dtype
 * A row whose page index is outside [0, num_pages), or beyond max_pages pages, is not copied;
 * slots that receive no row are left untouched. */
fc_status flashcache_select_gather_paged(const void* K, const void* V, const fc_kv_desc* desc,
                                         const float* scores, const int32_t* budgets,
                                         const int64_t* layer_offsets, int64_t rows_per_seq,
                                         int32_t shared, int32_t* idx_out, const int32_t* block_table,
                                         int32_t page_size, int32_t max_pages, int64_t num_pages,
                                         void* K_cache, void* V_cache, void* workspace,
                                         size_t workspace_bytes, void* hip_stream);

/* Decode-step attention over the compacted cache (Preliminary section, Eq. 2-4, for one new token
 * per sequence): for every (b, l) and query head g (q_heads = G * kv_heads; query head g reads
 * KV head g / G)   out[b][l][g] = softmax(q[b][l][g] . K_rows^T * scale) V_rows   over the b_l rows
 * that (b, l, g / G) kept.  Rows are read once, so the cost falls with the retention ratio.
 *   Q              device in, [B][L][q_heads][d], dtype per `dtype`
 *   K_cache/V_cache  device in, [B][rows_per_seq][d] packed as written by flashcache_select_gather
 *                  (an uncompressed [B][L][H][N][d] cache is the same layout with b_l = N)
 *   budgets, layer_offsets  device in, as written by flashcache_allocate
 *   out            device out, float [B][L][q_heads][d]; a unit with no rows gives zeros
 *   workspace      device, 16-byte aligned, flashcache_decode_workspace_bytes() bytes
 * Supported: d in {64, 128}; bf16 caches with any G from 1 to 16 (scores and weighted sums on the
 * matrix cores: bf16 products are exact in fp32, probabilities enter the second product as two
 * bf16 terms), fp32 caches with G in {1, 2, 4, 7, 8} (vector ALUs).  Accumulation in fp32; anything
 * else returns FC_EUNSUPPORTED. */
size_t flashcache_decode_workspace_bytes(int32_t batch, int32_t layers, int32_t kv_heads, int32_t q_heads,
                                         int32_t head_dim);
fc_status flashcache_decode_attention(const void* Q, const void* K_cache, const void* V_cache,
                                      int32_t batch, int32_t layers, int32_t kv_heads, int32_t q_heads,
                                      int32_t head_dim, int32_t dtype, const int32_t* budgets,
                                      const int64_t* layer_offsets, int64_t rows_per_seq, float scale,
                                      float* out, void* workspace, size_t workspace_bytes,
                                      void* hip_stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): flashcache_decode_attention without a workspace
 * argument.  The per-chunk partial results live in a fixed array inside the library's device image
 * (flashcache_decode_static_scratch_bytes() bytes, 16 MiB, held by every GPU the library runs on
 * until the process ends); the call allocates and frees nothing.  Arguments, results (bit for bit)
 * and errors are those of flashcache_decode_attention, except:
 *   - FC_EWORKSPACE if flashcache_decode_workspace_bytes() for the shape exceeds the array (nothing
 *     is enqueued);
 *   - all calls on one GPU share the array: two calls whose kernels overlap on that GPU (different
 *     streams without ordering between them) race on it.  Calls on one stream are safe; nothing has
 *     to be cleared between calls, every record that is read has been written by the same call. */
size_t flashcache_decode_static_scratch_bytes(void);
fc_status flashcache_decode_attention_static(const void* Q, const void* K_cache, const void* V_cache,
                                             int32_t batch, int32_t layers, int32_t kv_heads,
                                             int32_t q_heads, int32_t head_dim, int32_t dtype,
                                             const int32_t* budgets, const int64_t* layer_offsets,
                                             int64_t rows_per_seq, float scale, float* out,
                                             void* hip_stream);

/* The same attention over a paged cache, as written by flashcache_select_gather_paged: row j of unit
 * (b, l, h) is read from slot j % page_size of page block_table[b][l][h][j / page_size] of
 * K_pages / V_pages [num_pages][page_size][d].  Rows whose page entry is negative or >= num_pages
 * (never written) are not attended to; a unit without attended rows gives zeros.  budgets as
 * written by flashcache_allocate; workspace as for flashcache_decode_attention. */
fc_status flashcache_decode_attention_paged(const void* Q, const void* K_pages, const void* V_pages,
                                            const int32_t* block_table, int32_t page_size,
                                            int32_t max_pages, int64_t num_pages, int32_t batch,
                                            int32_t layers, int32_t kv_heads, int32_t q_heads,
                                            int32_t head_dim, int32_t dtype, const int32_t* budgets,
                                            float scale, float* out, void* workspace,
                                            size_t workspace_bytes, void* hip_stream);

/* Measurement aid (off by default; not part of the method).  While enabled, every kernel the
 * library launches is bracketed by a pair of HIP events on its launch stream.
 * flashcache_profile_enable(on) clears the records and switches recording on or off.
 * flashcache_profile_read waits for the recorded events and returns, per kernel name, the
 * launch count and the summed duration in milliseconds: `names` (host) receives up to
 * max_entries zero-terminated strings of name_stride bytes each, `launches` and `total_ms`
 * (host) the figures, *n_entries the number of distinct kernels seen. */
fc_status flashcache_profile_enable(int32_t on);
fc_status flashcache_profile_read(int32_t max_entries, char* names, int32_t name_stride,
                                  int32_t* launches, float* total_ms, int32_t* n_entries);

/* Static, human-readable name of a status code. */
const char* flashcache_status_string(int32_t status);

#ifdef __cplusplus
}
#endif
#endif /* FLASHCACHE_H_ */
