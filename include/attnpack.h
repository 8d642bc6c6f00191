/*
 * attnpack.h -- C ABI of the AttentionPack decode hot path for AMD MI355X (gfx950).
 *
 * A layer's KV cache K, V in R^{T x HD} (all H heads merged along the hidden
 * axis, HD = H*d; paper Sec. 3.1) is held as coefficient rows
 *     C_k, C_v  [T, r]      (the paper's compressed cache  Kbar, Vbar)
 * plus decompression matrices ("bases")
 *     B_k, B_v  [r, HD]     (the paper's D_k, D_v),
 * with K ~= C_k B_k, V ~= C_v B_v.  Head h owns hidden columns [h*d, (h+1)*d).
 * Grouped-query models (the paper's Sec. 4.5: fewer key/value heads than query
 * heads): the cache has H_kv heads, HD = H_kv*d, and query head h reads the
 * columns of key/value head h / (H / H_kv).  The decode calls take both H (query
 * heads) and H_kv; H_kv == H is ordinary multi-head attention.
 *
 * Conventions shared by every call
 *   - Every pointer is DEVICE memory owned by the caller unless marked "host".
 *     The library never allocates, frees or retains device memory.
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*; NULL =
 *     the default stream).  Calls return without synchronising; outputs are
 *     valid once the stream reaches that point.
 *   - The calls enqueue kernels only: no allocation, no memset, no synchronisation.  They may
 *     be captured in a HIP graph, provided a call with the same shapes has run once before the
 *     capture (the first launch of a kernel variant sets its shared-memory limit, which is not
 *     a stream operation) and timing (ap_prof_enable) is off.
 *   - Matrices are dense row-major.  Rows of C_k, C_v, B_k, B_v, K, V must start
 *     on 16-byte boundaries (true for r % 8 == 0 / HD % 8 == 0 in 2-byte types).
 *   - Errors are return codes; nothing is thrown or aborted.  Everything that can
 *     be checked on the host is rejected BEFORE any kernel is launched, and then
 *     no output is written.  ap_last_error() (thread-local, host string) says why.
 *     Device-side data errors (NaN mass, rank arrays that disagree with the bucket
 *     lists, ranks that are not multiples of the granularity) are undefined
 *     behaviour within the caller's buffers: documented, not checked.
 *   - State the library keeps per process (everything else lives in the caller's buffers):
 *     the records and switch of ap_prof_enable, the tuning value of
 *     ap_set_fused_value_min_bytes, one flag per kernel variant saying that its
 *     shared-memory limit has been raised (set on the variant's first launch), and the
 *     per-device address of the scratch buffer of ap_decode_attn_static.  The compute entry
 *     points may be called from several host threads at once as long as nobody calls
 *     ap_prof_enable / ap_prof_read / ap_set_fused_value_min_bytes meanwhile and timing is
 *     off (the flags and the address are written with the same value by whoever comes first).
 */
#ifndef ATTNPACK_H
#define ATTNPACK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  AP_OK = 0,
  AP_ERR_INVALID_ARG = 1, /* NULL pointer, non-positive or inconsistent size, misalignment */
  AP_ERR_UNSUPPORTED = 2, /* valid request outside what the kernels implement          */
  AP_ERR_WORKSPACE = 3,   /* workspace missing or smaller than the *_workspace_bytes query */
  AP_ERR_HIP = 4          /* the HIP runtime reported an error at launch                */
} ap_status;

typedef enum {
  AP_F32 = 0, /* IEEE binary32                                   */
  AP_F16 = 1, /* IEEE binary16                                   */
  AP_BF16 = 2, /* bfloat16 (upper half of a binary32)            */
  AP_I8 = 3,  /* signed 8-bit codes (coefficients only)          */
  AP_I4 = 4   /* 4-bit codes, two per byte (coefficients only)   */
} ap_dtype;

/* Columns per int8 scale (one fp16 scale per token per AP_QBLOCK columns). */
#define AP_QBLOCK 64

/* ------------------------------------------------------------------------
 * ap_compact -- multi-head compaction with given bases (paper Sec. 3.1:
 * Kbar = K D_k^T for D_k with orthonormal rows, i.e. U_r Sigma_r of the SVD).
 *
 *   Ck[b, row0 + i, :] = K[b, i, :] . Bk[b]^T      i = 0 .. n-1
 *   Cv[b, row0 + i, :] = V[b, i, :] . Bv[b]^T
 *
 * n = T is the prefill compression; n = 1 appends one decoded token's
 * coefficients to a cache whose basis is already fixed.
 *
 *   K, V     [B, n, HD]  dtype dt_in (AP_F16 | AP_BF16 | AP_F32), contiguous.
 *   Bk, Bv   [r, HD]     dtype dt_in; batch b uses Bk + b*basis_batch_stride
 *                        elements (0 = one basis shared by the whole batch).
 *   Ck, Cv   [B, T_cap, r] dtype dt_out, rows row0 .. row0+n-1 written.
 *            dt_out == dt_in, or AP_I8 (dt_in must then be AP_F16): the
 *            projection is rounded to fp16 first and then quantised per token
 *            and per AP_QBLOCK columns:  amax = max|c|; scale = fp16(fp32(amax) /
 *            127.0f); code = clamp(rint_even(fp32(c) / fp32(scale)), -127, 127),
 *            all zero when scale == 0.
 *   scale_k, scale_v  [B, T_cap, r / AP_QBLOCK] fp16; required iff dt_out == AP_I8.
 *   Accumulation is fp32; the result is rounded to nearest-even.
 *   Requires HD % 8 == 0, r % 16 == 0 (r % AP_QBLOCK == 0 for AP_I8),
 *   0 <= row0, row0 + n <= T_cap.  A K/V pair may be skipped by passing
 *   K == NULL (then Ck is untouched), likewise V.
 * ---------------------------------------------------------------------- */
ap_status ap_compact(const void* K, const void* V, const void* Bk, const void* Bv,
                     void* Ck, void* Cv, void* scale_k, void* scale_v,
                     int B, int n, int row0, int T_cap, int HD, int r,
                     int64_t basis_batch_stride, ap_dtype dt_in, ap_dtype dt_out,
                     void* stream);

/* ------------------------------------------------------------------------
 * ap_compute_bases -- the compression step itself (paper Sec. 3.1: low-rank SVD of
 * the head-merged cache; Alg. 1, compress step; the appendix's implementation
 * details: randomized SVD).  For every sequence b the rows of Bm[b] are the r
 * leading right singular vectors of X[b] (approximately: randomized range finder
 * on the row space with l = r + oversample vectors and power_iters power
 * iterations, then Rayleigh-Ritz), orthonormal, in decreasing order of singular
 * value, so that leading rows / coefficient columns carry the most energy.  The
 * coefficients then follow from ap_compact(X, Bm).
 *
 *   X      [B, n, HD]  dt (AP_F16 | AP_BF16), contiguous
 *   Omega  [l, HD]     dt: the start block (random numbers are the caller's: e.g.
 *                      i.i.d. Gaussian entries; any block of full row rank works);
 *                      sequence b reads Omega + b*omega_batch_stride elements
 *                      (0 = one block for all)
 *   Bm     [B, r, HD]  dt, written
 *   sigma  [B, r] fp32 or NULL: the singular values that go with the rows
 *   power_iters  0 .. 16; 2 is enough for spectra that decay like i^-0.7
 *   workspace    ap_bases_workspace_bytes(B, n, HD, r, oversample) bytes, 256-byte
 *                aligned (0 from the query = unsupported shape)
 * Requires HD % 64 == 0, n % 8 == 0, l even, l <= 1024, l <= n, l <= HD.
 * A basis is unique only up to the sign of each row (and rotations inside equal
 * singular values): results are to be judged by what they achieve (orthonormal
 * rows, residual of the rank-r reconstruction against the optimum), not compared
 * element by element.  Directions that X does not span (fewer than l independent
 * rows) come out as zero rows at the end of the order.
 *
 * ap_decompress -- Alg. 1 "retrieve cache" as a matrix:
 *   X[b, t, :] = C[b, t, :rank[b,t]] . Bm[b][:rank[b,t]]        t < T
 * i.e. what the periodic re-compression decomposes again, next to the uncompressed
 * tail: write it in front of the tail's rows, call ap_compute_bases and ap_compact
 * on the whole.
 *   C     [B, T_cap, r] dt;  Bm [r, HD] dt (+ basis_batch_stride, 0 = shared)
 *   rank  [B, T] int32 or NULL (= r everywhere)
 *   X     [B, T, HD] dt, written (fp32 accumulation, rounded to nearest even)
 *   workspace  ap_decompress_workspace_bytes(B, T, HD, r, rank != NULL), 256-byte aligned
 * Requires r % 64 == 0, HD % 8 == 0.
 * ---------------------------------------------------------------------- */
size_t ap_bases_workspace_bytes(int B, int n, int HD, int r, int oversample);
ap_status ap_compute_bases(const void* X, const void* Omega, int64_t omega_batch_stride,
                           void* Bm, float* sigma, int B, int n, int HD, int r, int oversample,
                           int power_iters, ap_dtype dt, void* workspace, size_t ws_bytes,
                           void* stream);
size_t ap_decompress_workspace_bytes(int B, int T, int HD, int r, int with_ranks);
ap_status ap_decompress(const void* C, const void* Bm, int64_t basis_batch_stride,
                        const int32_t* rank, void* X, int B, int T, int T_cap, int HD, int r,
                        ap_dtype dt, void* workspace, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * ap_quantize_i8 -- the int8 coefficient format of ap_compact applied to
 * coefficients that already exist in fp16 (same recipe, bit for bit).
 *   C      [B, T_cap, r] fp16, rows 0..T-1 read
 *   codes  [B, T_cap, r] int8, scales [B, T_cap, r / AP_QBLOCK] fp16
 * ---------------------------------------------------------------------- */
ap_status ap_quantize_i8(const void* C, void* codes, void* scales,
                         int B, int T, int T_cap, int r, void* stream);

/* ------------------------------------------------------------------------
 * ap_quantize_i4 -- 4-bit coefficients (paper Sec. 4.5 and Table 4 combine the
 * method with 4-bit quantisation of the cache; the reading taken for the format
 * is the uniform one, with the block structure of the int8 format): per token and
 * per AP_QBLOCK columns  amax = max|c|; scale = fp16(fp32(amax) / 7.0f);
 * code = clamp(rint_even(fp32(c) / fp32(scale)), -7, 7), all zero when scale == 0.
 * Two codes per byte: byte i of a row holds column 2i in its low nibble and column
 * 2i+1 in its high nibble, each nibble the code plus 8.
 *   C      [B, T_cap, r] fp16, rows 0..T-1 read
 *   codes  [B, T_cap, r / 2] bytes, scales [B, T_cap, r / AP_QBLOCK] fp16
 * ap_decode_attn reads the result with dt_coef = AP_I4 (dt = AP_F16): the codes
 * enter the matrix cores as exact integers, a coefficient's value is code * scale
 * with the scale applied in fp32, as for AP_I8.  Per-token ranks are multiples of
 * AP_QBLOCK.
 * ---------------------------------------------------------------------- */
ap_status ap_quantize_i4(const void* C, void* codes, void* scales,
                         int B, int T, int T_cap, int r, void* stream);

/* ------------------------------------------------------------------------
 * ap_select_ranks -- attention-aware rank groups (paper Sec. 3.2; Alg. 1,
 * group-selection step).
 *
 * Per batch row: tokens are ordered by (mass descending, token index
 * ascending); group g (0 = most important) takes sorted positions
 * [floor(T*cum_num[g-1]/den), floor(T*cum_num[g]/den)), cum_num[-1] := 0,
 * and its tokens are decoded at rank group_rank[g].
 *
 *   mass        [B, T] fp32, finite, >= 0 (the importance I of Eq. 1)
 *   group_rank  [F] HOST int32, non-increasing, each > 0 (not validated
 *               against any r here; ap_decode_attn validates what it is given)
 *   cum_num     [F] HOST int32, non-decreasing, cum_num[F-1] == den > 0
 *   rank_out    [B, T] int32: rank of every token
 *   bucket_off  [B, F+1] int32: group g's tokens are bucket_idx[b, off[g] .. off[g+1])
 *   bucket_idx  [B, T] int32: token indices, ascending inside each group
 *   workspace   >= ap_select_workspace_bytes(B, T, F) bytes, 16-byte aligned; its
 *               contents need not be preserved or cleared between calls (long rows
 *               in small batches are split over workgroups that meet there)
 * 1 <= F <= 8.  Results are unique, so they are comparable bit for bit.
 * ---------------------------------------------------------------------- */
ap_status ap_select_ranks(const float* mass, int B, int T, int F,
                          const int32_t* group_rank, const int32_t* cum_num, int32_t den,
                          int32_t* rank_out, int32_t* bucket_off, int32_t* bucket_idx,
                          void* workspace, size_t ws_bytes, void* stream);

size_t ap_select_workspace_bytes(int B, int T, int F);

/* ------------------------------------------------------------------------
 * ap_decode_attn -- one decode query per sequence attends to every cached
 * token of the compacted cache (paper Alg. 1: partial decompression, scores,
 * softmax, output; without the output projection W_o).
 *
 * Result (what the kernels compute, by associativity, without rebuilding K, V):
 *   Ktilde[t] = Ck[t, :rk_t] . Bk[:rk_t],  Vtilde[t] = Cv[t, :rv_t] . Bv[:rv_t]
 *   out[b,h]  = softmax_t( sm_scale * q[b,h] . Ktilde[t, head h] ) . Vtilde[:, head h]
 *   lse[b,h]  = log sum_t exp( sm_scale * q[b,h] . Ktilde[t, head h] )   (natural log)
 *
 *   q        [B, H, d] dtype dt
 *   Ck, Cv   [B, T_cap, r] dtype dt_coef (== dt, or AP_I8 / AP_I4 with dt == AP_F16;
 *            AP_I4 rows are r / 2 bytes);
 *            rows 0..T-1 are attended (no mask: the newest token is appended
 *            before attention, as in Alg. 1).
 *   scale_k, scale_v  [B, T_cap, r / AP_QBLOCK] fp16, required iff dt_coef is AP_I8 or AP_I4;
 *            a coefficient's value is code * scale.
 *   Bk, Bv   [r, H_kv*d] dtype dt, batch b at + b*basis_batch_stride elements (0 = shared)
 *   H_kv     key/value heads; must divide H.  With H_kv < H the fused step of
 *            ap_decode_step appends with a pass of its own over each basis.
 *   rank_k, rank_v  [B, T] int32 per-token ranks, or NULL = every token at rank r.
 *            One rank per token, shared by all heads.
 *   bucket_off [B, F+1], bucket_idx [B, T], F: the group lists ap_select_ranks
 *            produced for these rank arrays (every token of a group has the same
 *            rank_k and the same rank_v).  Required for AP_F16 / AP_BF16 when a rank
 *            array is given (the kernels walk rank-uniform token tiles); ranks must
 *            then be multiples of 16 in [16, r] (the paper's low ranks are 16 and 32),
 *            multiples of AP_QBLOCK = 64 with int8 coefficients (a scale block is read
 *            whole or not at all).  Other values are device-side data errors: a rank is
 *            then applied rounded down to a multiple of 8 (of 64 for int8), nothing is
 *            read out of bounds.  AP_F32 reads the rank arrays directly (any value in
 *            [0, r]) and ignores the bucket lists.
 *   out      [B, H, d] dtype dt_out: dt (round-to-nearest-even from fp32) or AP_F32.
 *            bfloat16 keeps 8 significant bits (unit roundoff 2^-8 = 3.9e-3), so a
 *            bf16 output cannot meet a 2e-3 error bound by rounding alone: callers
 *            that need the fp32 accumulator's accuracy ask for AP_F32.
 *   lse      [B, H] fp32 or NULL
 *   scores   [B, T_cap, H] fp32 or NULL: the scaled logits sm_scale * q[b,h] . Ktilde[t, head h]
 *            of the attended tokens (rows 0..T-1; with group lists only the listed tokens
 *            are written), for ap_update_importance.
 *   sm_scale softmax scale; pass 1/sqrt(d) for the paper's attention
 *   workspace >= ap_decode_workspace_bytes(...) bytes, 256-byte aligned.
 *
 * Supported shapes: AP_F32: anything (simple kernels, meant for small cases).
 * AP_F16 / AP_BF16: H <= 64, d in {32, 64, 128, 256}, r % 64 == 0, r <= 640.
 * Anything else returns AP_ERR_UNSUPPORTED.  1 <= T <= T_cap.
 * Scores, softmax and every accumulation are fp32 (the paper computes attention
 * in full precision over a half-precision cache).
 * ---------------------------------------------------------------------- */
ap_status ap_decode_attn(const void* q, const void* Ck, const void* Cv,
                         const void* scale_k, const void* scale_v,
                         const void* Bk, const void* Bv, int64_t basis_batch_stride,
                         const int32_t* rank_k, const int32_t* rank_v,
                         const int32_t* bucket_off, const int32_t* bucket_idx, int F,
                         void* out, float* lse, float* scores,
                         int B, int H, int H_kv, int d, int T, int T_cap, int r, float sm_scale,
                         ap_dtype dt, ap_dtype dt_coef, ap_dtype dt_out,
                         void* workspace, size_t ws_bytes, void* stream);

size_t ap_decode_workspace_bytes(int B, int H, int d, int T, int r, ap_dtype dt);

/* ------------------------------------------------------------------------
 * ap_decode_attn_static -- ap_decode_attn for callers that cannot allocate device
 * memory or carry a workspace around: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and the same
 * results as ap_decode_attn, but the split partials and the folded query live in a
 * buffer of AP_STATIC_SCRATCH_BYTES bytes that belongs to the library (a device
 * array in its code object, one copy per GPU, held until the process ends).  The
 * call allocates and frees nothing and calls no allocating routine.
 *   - A shape whose ap_decode_workspace_bytes() exceeds AP_STATIC_SCRATCH_BYTES is
 *     rejected with AP_ERR_WORKSPACE before any launch (the five benchmark shapes
 *     of this library fit; very long contexts at large batch do not).
 *   - Every call on a GPU uses that GPU's one buffer and finds the previous call's
 *     contents in it; nothing in it has to start at zero.  Two calls that overlap
 *     on one GPU (different streams, or different host threads without ordering)
 *     race on it: serialise them on one stream, or use ap_decode_attn.
 *   - The first call on a device looks the buffer's address up (not a stream
 *     operation): make it once before capturing a graph, as for every entry point.
 * ---------------------------------------------------------------------- */
#define AP_STATIC_SCRATCH_BYTES (64u << 20)
ap_status ap_decode_attn_static(const void* q, const void* Ck, const void* Cv,
                                const void* scale_k, const void* scale_v,
                                const void* Bk, const void* Bv, int64_t basis_batch_stride,
                                const int32_t* rank_k, const int32_t* rank_v,
                                const int32_t* bucket_off, const int32_t* bucket_idx, int F,
                                void* out, float* lse, float* scores,
                                int B, int H, int H_kv, int d, int T, int T_cap, int r, float sm_scale,
                                ap_dtype dt, ap_dtype dt_coef, ap_dtype dt_out, void* stream);

/* ------------------------------------------------------------------------
 * ap_decode_step -- one decode step with append (paper Alg. 1: the new token's
 * key and value join the cache, then the query attends to every cached token).
 * Computes what
 *     ap_compact(k_new, v_new, Bk, Bv, Ck, Cv, ..., n = 1, row0 = T - 1, ...)
 *     ap_decode_attn(q, Ck, Cv, ..., T, ...)
 * compute, but reads each basis once instead of twice: the key row's projection
 * shares its pass over B_k with the fold of the query, and the value row's
 * projection shares its pass over B_v with the expansion of the output, the new
 * token's own contribution being added there (limited to the basis rows below its
 * own value rank when per-token ranks are given).  The appended key
 * row has the same bits as ap_compact's; the value row and the outputs agree with
 * the two-call sequence up to the order of fp32 additions.
 *   k_new, v_new  [B, HD] dtype dt: the new token's merged-head key and value rows.
 *   Ck, Cv        [B, T_cap, r] dtype dt: row T-1 is WRITTEN, rows 0..T-1 attended.
 *   T             tokens cached after the append (1 <= T <= T_cap).
 * AP_F16 / AP_BF16 only (no int8 coefficients).  Rank arrays and group lists, when
 * given, must already cover the new token.
 * Everything else as ap_decode_attn; the workspace query is ap_decode_workspace_bytes.
 * ---------------------------------------------------------------------- */
ap_status ap_decode_step(const void* q, const void* k_new, const void* v_new, void* Ck, void* Cv,
                         const void* Bk, const void* Bv, int64_t basis_batch_stride,
                         const int32_t* rank_k, const int32_t* rank_v,
                         const int32_t* bucket_off, const int32_t* bucket_idx, int F,
                         void* out, float* lse, float* scores,
                         int B, int H, int H_kv, int d, int T, int T_cap, int r, float sm_scale,
                         ap_dtype dt, ap_dtype dt_out,
                         void* workspace, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * ap_update_importance -- the paper's importance update (Eq. 1) for one new
 * query (T_q = 1), from the logits and log-sum-exp a decode call returned:
 *     A[b,h,t]   = exp(scores[b,t,h] - lse[b,h])             attention weights
 *     mass[b,t] <- alpha * mass[b,t] + (1 - alpha) * mean_h A[b,h,t]     t < T
 *   scores  [B, T_cap, H] fp32, lse [B, H] fp32 (natural log), as written by
 *           ap_decode_attn / ap_decode_step with all T tokens attended
 *   mass    [B, mass_stride] fp32, updated in place; a token that has just been
 *           appended should enter with mass 0 (the caller's initialisation)
 *   0 <= alpha <= 1.  The result feeds ap_select_ranks.
 * ---------------------------------------------------------------------- */
ap_status ap_update_importance(const float* scores, const float* lse, float* mass,
                               int B, int H, int T, int T_cap, int64_t mass_stride,
                               float alpha, void* stream);

/* ------------------------------------------------------------------------
 * The uncompressed segment of the cache (Alg. 1: C_u = {K, V}; in the paper's
 * experiments the text tokens, and every generated token until the next
 * compression) and the merge of segments under one softmax.
 *
 * ap_raw_attn -- softmax attention of one decode query per sequence over raw
 * keys and values:  out[b,h,:] = softmax_t(sm_scale q[b,h].K[b,t,head h]) V[b,t,head h]
 *   q    [B, H, d]          dt (fp16 or bf16)
 *   K, V [B, T_u_cap, H_kv*d]  dt; rows 0..T_u-1 are attended; query head h reads
 *        the columns of key/value head h / (H / H_kv)
 *   out  [B, H, d] fp32; lse [B, H] fp32 natural log-sum-exp of the scaled
 *        logits, or NULL.  T_u = 0 gives out = 0 and lse = -inf.
 *   d in {32, 64, 128, 256}; workspace of ap_raw_workspace_bytes(B, H, d, T_u).
 *
 * ap_merge_segments -- attention over two disjoint token sets to attention over
 * their union (Alg. 1 concatenates the decompressed and the uncompressed tokens
 * before the softmax; the softmax of a concatenation is the mean of the
 * per-segment results weighted by exp(lse_i)):
 *     w_i = exp(lse_i - max(lse_a, lse_b)),  out = (w_a out_a + w_b out_b) / (w_a + w_b),
 *     lse = max + log(w_a + w_b)
 *   out_a, out_b [B, H, d] fp32 (e.g. from ap_decode_attn with dt_out = AP_F32 and
 *   from ap_raw_attn), lse_a, lse_b [B, H] fp32; out [B, H, d] in dt_out (may be
 *   out_a or out_b itself when dt_out is AP_F32), lse [B, H] or NULL (a buffer of
 *   its own: not lse_a or lse_b).  A segment with lse = -inf drops out.  More than
 *   two segments: call repeatedly.
 *
 * ap_raw_append -- k_new, v_new [B, HD] (either may be NULL) copied to row `row`
 * of K, V [B, T_u_cap, HD].
 * ---------------------------------------------------------------------- */
size_t ap_raw_workspace_bytes(int B, int H, int d, int T_u);
ap_status ap_raw_attn(const void* q, const void* K, const void* V, float* out, float* lse,
                      int B, int H, int H_kv, int d, int T_u, int T_u_cap, float sm_scale,
                      ap_dtype dt, void* workspace, size_t ws_bytes, void* stream);
ap_status ap_merge_segments(const float* out_a, const float* lse_a,
                            const float* out_b, const float* lse_b,
                            void* out, float* lse, int B, int H, int d,
                            ap_dtype dt_out, void* stream);
ap_status ap_raw_append(const void* k_new, const void* v_new, void* K, void* V,
                        int B, int HD, int row, int T_u_cap, ap_dtype dt, void* stream);

/* ------------------------------------------------------------------------
 * ap_keyonly_attn -- decode attention over a cache whose KEYS are compressed
 * while its values are kept as they are (paper appendix "Analysis of Textual
 * Token Compression", the text-domain experiment:
 * values need a higher rank than keys there, so only the keys are compressed,
 * R_k = 64).  The same segment algebra as above applies: keys Ktilde = Ck Bk,
 *
 *   out[b, h] = softmax_t( sm_scale * q[b, h] . Ktilde[b, t, slice(h)] ) V[b, t, slice(h)]
 *
 * computed with the basis folded into the query (q' = Bk[:, slice] q, one dot
 * product of length r per token and head instead of a rebuilt key).
 *
 *   q        [B, H, d]           dt (AP_F16 | AP_BF16)
 *   Ck       [B, T_cap, r]       dt, rows 0 .. T-1 read
 *   Bk       [r, H_kv*d]         dt; batch b uses Bk + b*basis_batch_stride elements (0 = shared)
 *   V        [B, T_cap, H_kv*d]  dt, rows 0 .. T-1 read (same T_cap as Ck)
 *   out      [B, H, d] fp32; lse [B, H] fp32 natural-log sum of exponentials, or NULL.
 *            T == 0 gives out = 0, lse = -inf.  (out, lse) can be joined with other
 *            segments by ap_merge_segments.
 *   workspace  ap_keyonly_workspace_bytes(B, H, H_kv, d, T, r) bytes, 256-byte aligned
 *            (0 from the query = unsupported shape).
 *   Requires d in {32, 64, 128, 256}, r % 8 == 0, r <= 640, H % H_kv == 0.
 *   A generated token is added with ap_compact (K only, n = 1) and ap_raw_append
 *   (v_new only).
 * ---------------------------------------------------------------------- */
size_t ap_keyonly_workspace_bytes(int B, int H, int H_kv, int d, int T, int r);
ap_status ap_keyonly_attn(const void* q, const void* Ck, const void* Bk,
                          int64_t basis_batch_stride, const void* V,
                          float* out, float* lse, int B, int H, int H_kv, int d,
                          int T, int T_cap, int r, float sm_scale, ap_dtype dt,
                          void* workspace, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * ap_valueonly_attn -- the mirror image: keys kept as they are, VALUES
 * compressed (Vtilde = Cv Bv; the other one-sided variant, which the same
 * appendix passage sets aside because values need the higher rank):
 *
 *   out[b, h] = softmax_t( sm_scale * q[b, h] . K[b, t, slice(h)] ) Vtilde[b, t, slice(h)]
 *
 * computed as (sum_t p[h, t] Cv[t, :]) Bv[:, slice(h)]: the weighted sum runs over
 * coefficient rows, the basis is applied once at the end.
 *
 *   q        [B, H, d]           dt (AP_F16 | AP_BF16)
 *   K        [B, T_cap, H_kv*d]  dt, rows 0 .. T-1 read
 *   Cv       [B, T_cap, r]       dt (same T_cap)
 *   Bv       [r, H_kv*d]         dt; batch b uses Bv + b*basis_batch_stride elements (0 = shared)
 *   out      [B, H, d] fp32; lse [B, H] fp32 or NULL.
 *   workspace  ap_valueonly_workspace_bytes(B, H, H_kv, d, T, r) bytes, 256-byte aligned
 *            (0 from the query = unsupported shape).
 *   Requires T >= 1, d in {32, 64, 128, 256}, r % 8 == 0, r <= 640 (320 at d = 32),
 *   H % H_kv == 0, H_kv*d <= 8192.  A generated token is added with ap_raw_append
 *   (k_new only) and ap_compact (V only, n = 1).
 * ---------------------------------------------------------------------- */
size_t ap_valueonly_workspace_bytes(int B, int H, int H_kv, int d, int T, int r);
ap_status ap_valueonly_attn(const void* q, const void* K, const void* Cv, const void* Bv,
                            int64_t basis_batch_stride, float* out, float* lse,
                            int B, int H, int H_kv, int d, int T, int T_cap, int r,
                            float sm_scale, ap_dtype dt, void* workspace,
                            size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Tuning of ap_decode_step (same results either way, up to fp32 summation
 * order).  A fused step can produce the new value row inside
 * its expansion pass over B_v (B_v is then read once per step; the pass writes
 * per-row-block sums that a small extra kernel adds up), or append it in a pass
 * of its own that runs in the same launch as the key row's (B_v is read twice,
 * one launch less).  The library takes the first way when the value bases
 * streamed per step, B * r * H_kv * d * 2 bytes (without the factor B when the
 * bases are shared), reach 128 MiB, or 96 MiB at r >= 512 (paper Alg. 1 fixes
 * the result, not the schedule).  min_bytes >= 0 replaces that rule by "at
 * least min_bytes" (0: always, a huge value: never); a negative value restores
 * it.  Process-wide, not thread-safe; meant for tests and tuning.
 * ---------------------------------------------------------------------- */
void ap_set_fused_value_min_bytes(int64_t min_bytes);

/* ------------------------------------------------------------------------
 * Timing of the dominant kernel (measurement aid, not part of the method).
 * While enabled, every ap_decode_attn / ap_decode_step call on AP_F16 / AP_BF16
 * attaches a pair of HIP events to the launch of its coefficient-streaming
 * kernel (hipExtLaunchKernelGGL: the events carry that kernel's own start and
 * end, not the gap to the kernel before it, so the time is the one a kernel
 * trace reports).  ap_prof_read waits for the last pair and returns the summed
 * kernel time in milliseconds and the number of pairs since ap_prof_enable(1),
 * which also clears the records.  ap_prof_enable(n) with n > 1 times every n-th
 * launch only (the first, the (n+1)-th, ...): the events cost a few microseconds
 * of pipeline bubble per timed launch, which a throughput measurement running
 * at the same time would otherwise pay on every step; ap_prof_enable(0) is off.  At most 4096 launches are recorded (later ones are
 * not timed).  Events are host-side handles owned by the library; no device
 * memory is allocated.  Not thread-safe.
 * ---------------------------------------------------------------------- */
void ap_prof_enable(int on);
ap_status ap_prof_read(float* total_ms, int* launches);
/* The same records one by one: waits for the last pair, writes the kernel time of the first
 * min(*launches, cap) timed launches to us[] (HOST array, microseconds, in launch order; -1 for
 * a pair that could not be read) and the number of pairs recorded to *launches. */
ap_status ap_prof_read_launches(float* us, int cap, int* launches);

/* ------------------------------------------------------------------------
 * Streaming-read yardstick (measurement aid, not part of the method).
 * ap_probe_read enqueues one kernel that reads `bytes` bytes from src with
 * plain 16-byte loads (2048 workgroups, eight loads in flight per thread) and
 * writes the XOR of what each wave read to sink; timing it gives the read bandwidth a kernel
 * can actually reach on this machine, next to which the bandwidth-bound
 * kernels of the library are reported.
 *   src    device buffer of at least `bytes` bytes, 16-byte aligned
 *   bytes  positive multiple of ap_probe_read_granule()
 *   sink   device buffer of 8192 uint32 (32 KiB), overwritten
 * ap_probe_read_stream is the same kernel with the non-temporal hint on its loads
 * (data that is read once): on MI355X it reads about 15 % faster, and it is the
 * yardstick for the kernels of the library that stream with that hint.
 * ---------------------------------------------------------------------- */
size_t ap_probe_read_granule(void);
ap_status ap_probe_read(const void* src, size_t bytes, void* sink, void* stream);
ap_status ap_probe_read_stream(const void* src, size_t bytes, void* sink, void* stream);

/* Host strings; ap_last_error() is thread-local and describes the most recent
 * non-AP_OK return on the calling thread ("" if none). */
const char* ap_status_string(ap_status s);
const char* ap_last_error(void);
/* Library version as major*10000 + minor*100 + patch. */
int ap_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ATTNPACK_H */
