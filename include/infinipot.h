/*
 * libinfinipot - the compression step of InfiniPot's Continual Context Distillation (CCD),
 * hand-written HIP for AMD MI355X (gfx950).
 *
 * When the fixed-size KV "memory pot" is full (paper Sec. 3.2), every unit - one (sequence b,
 * layer l, KV head h) triple - is compressed independently from n cached tokens to k = |C|:
 *
 *   score    representative score of Eq. 2: sum over the |P| catalyst-prompt (CaP) query tokens of
 *            their attention probability on each cached token (App. B, "Calculate Attention Score"),
 *            summed over the G = Hq/Hkv query heads that share the KV head; then 1-D pooling along
 *            the token axis; then the T tokens with the largest Novelty-under-Compression score
 *            (Eq. 3-4, passed in as `novelty`) are lifted to +inf (Sec. 3.3.3, App. B "Combine NuC
 *            and CaP").
 *   select   the k tokens with the largest score per unit (App. B "Final Token Selection"); equal
 *            scores go to the lower token index; indices are emitted in ascending order so the
 *            temporal order of the cache is preserved.
 *   compact  K' = K[keep_idx], V' = V[keep_idx] (App. B, the two gathers) - bit copies.
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers (HIP global memory) owned by the caller; the library
 *     never allocates, frees or keeps them.  `shape` is a HOST pointer, read during the call only.
 *   - `hip_stream` is a hipStream_t (NULL = the default stream).  Calls only enqueue kernels on that
 *     stream and return; nothing is synchronised and nothing is copied to the host.
 *   - Q_cat, K, V share `dtype` (fp32, or bf16 stored as 16-bit patterns).  The last dimension (d) is
 *     contiguous and the token / query-token dimension has stride d; the outer three dimensions use
 *     the strides in the shape (in elements).  Base pointers must be 16-byte aligned and the strides
 *     multiples of 16 bytes.
 *   - Return value: CCD_OK, CCD_NOOP (ccd_compress only) or a negative CCD_E* code.  All argument
 *     checks happen on the host before anything is launched; on an error nothing is launched and no
 *     buffer is touched.  Errors inside asynchronous kernels are not reported.
 */
#ifndef INFINIPOT_H
#define INFINIPOT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CCD_API __attribute__((visibility("default")))

enum {
  CCD_OK = 0,
  CCD_NOOP = 1,          /* pot not full (n_valid < n_cap) or nothing to drop (n_valid <= k): untouched */
  CCD_EINVAL = -1,       /* NULL pointer, or a shape field out of range                                 */
  CCD_EUNSUPPORTED = -2, /* d not in {64, 128}, unknown dtype or pool_mode, n_valid > 65536, a matrix-  */
                         /* core score_path that an fp32 cache cannot take (see score_path), or one     */
                         /* named for a window with P > 1986                                            */
  CCD_EALIGN = -3,       /* pointer or stride not 16-byte aligned                                       */
  CCD_EWORKSPACE = -4,   /* workspace NULL, misaligned or smaller than ccd_workspace_bytes()            */
  CCD_ELAUNCH = -5       /* the HIP runtime refused a kernel launch                                    */
};

enum { CCD_FP32 = 0, CCD_BF16 = 1 };
enum { CCD_POOL_NONE = 0, CCD_POOL_MAX = 1, CCD_POOL_AVG = 2 };
enum { CCD_PATH_AUTO = 0, CCD_PATH_VALU = 1, CCD_PATH_MFMA_SLICES = 2, CCD_PATH_MFMA_UNIT = 3 };

typedef struct {
  int32_t B, L, Hq, Hkv, d;   /* sequences, layers, query heads, KV heads (Hq % Hkv == 0), head dim      */
  int32_t n_valid;            /* n: tokens now in the pot, scored and selected from                      */
  int32_t n_cap;              /* capacity of the pot in tokens (paper: |M| - |P|); n_valid <= n_cap      */
  int32_t k;                  /* |C|: tokens kept, 1 <= k <= n_valid                                     */
  int32_t P;                  /* |P|: CaP query tokens per query head, >= 1                              */
  int32_t T;                  /* NuC slots, 0 <= T <= k (paper: alpha * |C|)                             */
  int32_t pool_w, pool_mode;  /* odd window >= 1; CCD_POOL_*.  max: window clipped at the ends;          */
                              /* avg: zero padding, divide by pool_w.  Pooling precedes the NuC lift.    */
  int32_t dtype;              /* CCD_FP32 or CCD_BF16, for Q_cat, K and V                                */
  float scale;                /* logit scale; 0 means 1/sqrt(d)                                          */
  int32_t window;             /* sliding attention window in tokens, 0 = none (Sec. 4, footnote on SWA   */
                              /* models): the cached tokens stand at positions 0 .. n_valid-1 and CaP    */
                              /* token i at n_valid + i; a query at position p sees the keys at          */
                              /* p-window+1 .. p only.  window >= P when set.  (The matrix-core score     */
                              /* paths take P <= 1986 under a window; beyond that CCD_PATH_AUTO scores on */
                              /* the vector ALUs and a matrix-core path that was named is refused.)       */
  int32_t score_path;         /* kernels for Eq. 2: CCD_PATH_AUTO (0) unless two paths are to be compared:       */
                              /* CCD_PATH_VALU vector ALUs; CCD_PATH_MFMA_SLICES (bf16 caches only) matrix       */
                              /* cores, a workgroup per token slice; CCD_PATH_MFMA_UNIT matrix cores, a          */
                              /* workgroup per unit.  All give the same scores up to fp32 rounding order.        */
                              /* fp32 caches on CCD_PATH_MFMA_UNIT: every fp32 value enters as the sum of two    */
                              /* bf16 values and a product as three bf16 products (scores within 1e-3 for        */
                              /* logits up to about 140, measured; 4e-4 at 65); d = 64 only, no window, no K_cap  */
                              /* (CCD_EUNSUPPORTED otherwise; CCD_PATH_AUTO then takes the vector ALUs).          */
  int64_t kv_stride_b, kv_stride_l, kv_stride_h;    /* K, V: [B, L, Hkv, n_cap, d], strides in elements */
  int64_t q_stride_b, q_stride_l, q_stride_h;       /* Q_cat: [B, L, Hq, P, d]                          */
  int64_t nov_stride_b, nov_stride_l, nov_stride_h; /* novelty fp32: [B, n] shared by layers and heads  */
                              /* when the l and h strides are both 0, else carried per head              */
                              /* [B, L, Hkv, n_cap].                                                     */
} ccd_shape_t;

/* Bytes of scratch that ccd_score and ccd_compress need for this shape (0 if the shape is invalid).
 * The workspace must be 256-byte aligned; its contents need not survive between calls. */
CCD_API size_t ccd_workspace_bytes(const ccd_shape_t* shape);

/* The score step (Eq. 2, pooling, Sec. 3.3.3 step 1): writes the final fp32 score of every token,
 * scores[B, L, Hkv, n_valid] (dense).  NuC-selected tokens hold +inf; finite scores whose magnitude
 * is below FLT_MIN are written as 0.  Tokens whose novelty is NaN or -inf never take a NuC slot. */
CCD_API int ccd_score(const ccd_shape_t* shape, const void* Q_cat, const void* K, const float* novelty,
              float* scores, void* workspace, size_t workspace_bytes, void* hip_stream);

/* Filling the pot (Sec. 3.2: new context is cached until the pot is full): rows n_valid .. n_valid + count - 1 of
 * every unit of K and V (layout and strides of the shape) take the rows of a chunk of new context, K_new and V_new
 * [B, L, Hkv, count, d], dense, cache dtype; requires n_valid + count <= n_cap (CCD_EINVAL otherwise; n_valid may
 * be 0, count may be 0).  novelty / novelty_new (both or neither): entries n_valid .. n_valid + count - 1 of
 * novelty (strides of the shape: shared [B, n], or carried per head [B, L, Hkv, n_cap], then every head gets them)
 * take novelty_new [B, count] fp32.  The caller raises n_valid by count afterwards.  Only B, L, Hkv, d, dtype,
 * n_valid, n_cap and the K/V and novelty strides of the shape are read.  (A model that writes its new keys and
 * values straight into the pot's free rows needs no such copy.) */
CCD_API int ccd_append(const ccd_shape_t* shape, void* K, void* V, float* novelty, const void* K_new, const void* V_new,
                       const float* novelty_new, int32_t count, void* hip_stream);

/* The select step (Sec. 3.3.3 step 2): keep_idx[B, L, Hkv, k] int32 = the k indices of largest score per unit,
 * ascending.  Equal scores: lower index first; NaN ranks with -inf; -0 equals +0.  Only B, L, Hkv,
 * n_valid and k of the shape are read. */
CCD_API int ccd_select(const ccd_shape_t* shape, const float* scores, int32_t* keep_idx, void* hip_stream);

/* The compact step (App. B gathers): row j of K_dst/V_dst (same layout and strides as the sources) becomes row
 * keep_idx[j] of K_src/V_src for j < k; rows >= k of the destination are left as they are.  K_dst may
 * equal K_src and V_dst may equal V_src (in place; keep_idx must be strictly ascending per unit, as
 * ccd_select produces); partially overlapping buffers are not allowed.  If `novelty_inout` is not NULL
 * and the shape carries per-head novelty, its first k entries per unit are compacted the same way. */
CCD_API int ccd_compact(const ccd_shape_t* shape, const void* K_src, const void* V_src, const int32_t* keep_idx,
                void* K_dst, void* V_dst, float* novelty_inout, void* hip_stream);

/* The fused step: score, select and compact K, V (and per-head novelty) in place.  Returns CCD_NOOP and
 * launches nothing when the pot is not full (Sec. 3.2: distillation happens once the cache is full).
 * keep_idx[B, L, Hkv, k] is always written; scores_opt[B, L, Hkv, n_valid] only if not NULL.  After
 * CCD_OK the caller's pot holds k tokens per unit; rows >= k are stale. */
CCD_API int ccd_compress(const ccd_shape_t* shape, const void* Q_cat, void* K, void* V, float* novelty,
                 float* scores_opt, int32_t* keep_idx, void* workspace, size_t workspace_bytes,
                 void* hip_stream);

/* ccd_compress for callers that cannot allocate device memory - code under HIP graph capture, serving loops that have
 * handed all memory out, harnesses that forbid hipMalloc: the workspace is a buffer of CCD_NOALLOC_WORKSPACE_BYTES that
 * the library itself holds on every GPU, from load to process end.  Same arguments, results and return codes as
 * ccd_compress, minus the workspace; shapes whose ccd_workspace_bytes() exceeds the buffer return CCD_EWORKSPACE and
 * nothing is launched.  Allocates nothing (the first call on a GPU looks the buffer's address up once).  All calls on
 * one GPU share the one buffer, whose contents are scratch and need not start at any value: calls that overlap in time
 * on the same GPU (two streams, two threads) race; on different GPUs they do not. */
#define CCD_NOALLOC_WORKSPACE_BYTES (16u << 20)
CCD_API int ccd_compress_noalloc(const ccd_shape_t* shape, const void* Q_cat, void* K, void* V, float* novelty,
                         float* scores_opt, int32_t* keep_idx, void* hip_stream);

/* NuC score from the model's logits (Sec. 3.3.2, Eq. 3; App. B "Calculate NuC Score"): the novelty of a token is its
 * cross entropy under the model, novelty[r] = log(sum_v exp(logits[r][v])) - logits[r][labels[r]], r < rows.
 * logits: device, [rows, V] of `dtype` (CCD_FP32 or CCD_BF16), rows `row_stride` elements apart (row_stride >= V, a
 * multiple of 16 bytes; base 16-byte aligned); row r must be the prediction FOR labels[r] (the caller shifts).
 * labels: device int32 [rows]; a label outside [0, V) marks a token without a prediction and gives -inf, which never
 * takes a NuC slot.  novelty: device fp32 [rows], the `novelty` input of ccd_score / ccd_compress.  fp32 arithmetic;
 * rows holding +inf or NaN logits give NaN.  rows == 0 returns CCD_OK and launches nothing. */
CCD_API int ccd_nuc_from_logits(const void* logits, const int32_t* labels, float* novelty, int64_t rows, int32_t V,
                        int64_t row_stride, int32_t dtype, void* hip_stream);

/* CR-RoPE (Sec. 3.5).  The pot stores keys BEFORE the rotary position embedding; after a distillation the kept
 * keys are embedded at their NEW positions 0 .. |C|-1.  ccd_cr_rope writes, for every unit, K_rot[j] = the rotary
 * embedding at position j of row j of K, for j < count (0 <= count <= n_cap); rows >= count of K_rot are left as they
 * are.  K_rot has the layout and strides of K and must not be K.  rope_cos and rope_sin are fp32 device tables
 * [>= count, d/2], dense (row stride d/2), 16-byte aligned: entry [p, i] is the cosine / sine of the angle of position
 * p for the pair (i, i + d/2): y_i = x_i cos - x_{i+d/2} sin, y_{i+d/2} = x_{i+d/2} cos + x_i sin (the caller's rope
 * base and scaling are in the tables).  Computed in fp32, rounded once to the cache's type (bf16: nearest even).
 * Only B, L, Hkv, d, n_valid, n_cap, k, dtype and the kv strides of the shape are read. */
CCD_API int ccd_cr_rope(const ccd_shape_t* shape, const void* K, const float* rope_cos, const float* rope_sin,
                int32_t count, void* K_rot, void* hip_stream);

/* ccd_compress with CR-RoPE in the same pass: as ccd_compress, and K_rot[j] = the rotary embedding at position j of
 * the j-th kept key, j < k (tables with at least k rows).  The pot itself (K) keeps the un-embedded keys.  K_rot must
 * not be NULL, K or V.  K_score (nullable; layout and strides of K): the keys the catalyst queries attend to when they
 * are not the stored ones - the model attends to the EMBEDDED keys of the current positions 0 .. n_valid-1, i.e. to the
 * attention cache that the previous call left in K_rot and the prefill extended; NULL scores on K itself.  K_score is
 * only read, and only before K_rot is written, so K_score may be the same buffer as K_rot.  K_cap (nullable): the CaP
 * tokens' own keys as in ccd_score_kcat below, embedded like K_score; lse (nullable, not together with K_cap): the rows'
 * log-sum-exps as in ccd_score_lse below.  On CCD_NOOP nothing is written, K_rot included. */
CCD_API int ccd_compress_rope(const ccd_shape_t* shape, const void* Q_cat, void* K, void* V, float* novelty,
                      float* scores_opt, int32_t* keep_idx, const void* K_score, const void* K_cap, const float* lse,
                      const float* rope_cos, const float* rope_sin, void* K_rot, void* workspace,
                      size_t workspace_bytes, void* hip_stream);

/* Eq. 2 read as the model's own (causal) attention row: the CaP tokens stand at the end of the sequence, so CaP token
 * i attends to the cached tokens AND to the CaP keys 0 .. i, which take their share of the probability mass; the
 * representative score still sums the cached tokens' columns only (App. B slices the CaP columns off).  ccd_score and
 * ccd_compress normalise over the cached tokens alone; these two take the CaP keys as well.
 * K_cap: device, [B, L, Hkv, P, d] dense (no strides), of the cache's dtype, 16-byte aligned, only read; must not be
 * NULL (CCD_EINVAL) nor alias K, V.  Everything else as in ccd_score / ccd_compress; same workspace. */
CCD_API int ccd_score_kcat(const ccd_shape_t* shape, const void* Q_cat, const void* K, const void* K_cap,
                   const float* novelty, float* scores, void* workspace, size_t workspace_bytes, void* hip_stream);
CCD_API int ccd_compress_kcat(const ccd_shape_t* shape, const void* Q_cat, void* K, void* V, const void* K_cap,
                      float* novelty, float* scores_opt, int32_t* keep_idx, void* workspace, size_t workspace_bytes,
                      void* hip_stream);

/* Eq. 2 with the normalisers handed in.  The model that ran the CaP tokens already normalised their attention rows; its
 * attention kernel returns, next to its output, the log-sum-exp of every row.  Given those, the probability of CaP
 * query (g, i) on cached token t is exp(scale * <q, k_t> - lse[g, i]) and the statistics pass over K is not needed: one
 * pass instead of two.  The normalisers cover whatever keys the model let the row attend to (the CaP tokens' own keys,
 * a sliding window), so this is the model's causal attention row of ccd_score_kcat without K_cap; shape.window still
 * says which cached tokens a row does NOT see (their probability is 0).
 * lse: device fp32 [B, L, Hq, P] dense, natural logarithm, of the logits scale * <q, k> (scale as in the shape),
 * 16-byte aligned, only read; must not be NULL (CCD_EINVAL).  Everything else as in ccd_score / ccd_compress; same
 * workspace. */
CCD_API int ccd_score_lse(const ccd_shape_t* shape, const void* Q_cat, const void* K, const float* lse, const float* novelty,
                  float* scores, void* workspace, size_t workspace_bytes, void* hip_stream);
CCD_API int ccd_compress_lse(const ccd_shape_t* shape, const void* Q_cat, void* K, void* V, const float* lse, float* novelty,
                     float* scores_opt, int32_t* keep_idx, void* workspace, size_t workspace_bytes, void* hip_stream);

/* Per-kernel timing of ccd_compress for benchmarks: a host-side aid, off by default, and the only state the library
 * keeps between calls (process-wide: enable it from one thread, for calls on one stream).  While enabled, each
 * kernel of ccd_compress is launched with two HIP events attached that take the kernel's own begin and end time
 * stamps (hipExtLaunchKernel; events are created on demand and reused; nothing is put into the stream between the
 * kernels and nothing else changes).  ccd_profile_collect waits for those
 * events, adds up the elapsed milliseconds per stage into stage_ms[ccd_profile_stages()] (host array) and stores
 * the number of calls covered in *calls (host), then forgets them.  Stage i is named ccd_profile_stage_name(i).
 * Not thread safe; meant for one stream. */
CCD_API int ccd_profile_enable(int on);
CCD_API int ccd_profile_stages(void);
CCD_API const char* ccd_profile_stage_name(int stage);
CCD_API int ccd_profile_collect(double* stage_ms, int64_t* calls);

/* Static, human-readable text for a return code. */
CCD_API const char* ccd_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* INFINIPOT_H */
