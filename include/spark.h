/*
 * spark.h -- C ABI of the MI355X (gfx950) Spark-FFN sparse decode library.
 *
 * The library evaluates the sparse feed-forward layer of the Spark Transformer
 * (arXiv 2506.06644):
 *
 *   Spark-FFN(q; K1, K2, V, k, r) = V * ( GELU( StatTop_k(K1^T q[:r]) ) (.) (K2^T q[r:]) )     Eq.2
 *   StatTop_k(x)   = max(x - theta, 0)                                                       Eq.9-10
 *   theta(x, k)    = mean(x) + std(x) * Q(1 - k/d),  std with 1/(d-1)                        Eq.11
 *
 * as the decode pipeline of Section 2.1 / Appendix B: predictor GEMV over the first r input
 * dimensions, statistical top-k, compaction of the active neurons, gathered GEMVs over only
 * the active rows of K2 and V.
 *
 * General conventions
 *   - All array arguments are DEVICE pointers (HIP global memory of the current device)
 *     unless the comment says "host".  The library never allocates or frees device memory:
 *     every buffer, including the workspace, is owned by the caller, and the workspace needs
 *     no initialisation.  No state is kept between calls: nothing a call does depends on an
 *     earlier call, and calls from several threads (on their own streams and workspaces) do
 *     not interact.
 *   - Calls enqueue work on `hip_stream` (a hipStream_t passed as void*; NULL = the default
 *     stream) and return without synchronising.  Outputs are valid once the stream has
 *     been synchronised by the caller.  Two calls that share a workspace must be ordered
 *     on one stream.
 *   - Arguments are validated on the host before anything is launched; an invalid call
 *     returns an error code and touches no memory.  Nothing throws or aborts across the ABI.
 *   - Weights are "neuron-major": row j of K1n / K2n / Vn is column j of the paper's
 *     K1 / K2 / V, so the data of one neuron is one contiguous burst.
 *   - Base pointers of weights, q and x must be 16-byte aligned and every row must span a
 *     multiple of 16 bytes (SPARK_ERR_ALIGN otherwise).
 */
#ifndef SPARK_H_
#define SPARK_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SPARK_VERSION 100
#define SPARK_MAX_BATCH 64 /* tokens per spark_ffn_decode call (the paper's prefill chunk) */

typedef enum {
  SPARK_OK = 0,
  SPARK_ERR_NULL = 1,      /* a required pointer is NULL                                    */
  SPARK_ERR_SHAPE = 2,     /* a dimension / stride / batch is out of range                  */
  SPARK_ERR_K = 3,         /* k outside [1, d-1] (the range of Theorem 1)                   */
  SPARK_ERR_DTYPE = 4,     /* unknown or unsupported dtype combination                      */
  SPARK_ERR_ALIGN = 5,     /* pointer or row pitch not 16-byte aligned                      */
  SPARK_ERR_WORKSPACE = 6, /* workspace NULL or smaller than the matching *_workspace_bytes */
  SPARK_ERR_DEVICE = 7     /* the HIP runtime refused a launch or a query                   */
} spark_status;

/* SPARK_FP8_E4M3 and SPARK_INT8 are weight types only (spark_ffn_layer.wdtype), one byte per
 * code: OCP E4M3 (1 sign, 4 exponent bits with bias 7, 3 mantissa bits, largest finite value
 * 448), or a signed integer in two's complement. */
typedef enum { SPARK_F32 = 0, SPARK_BF16 = 1, SPARK_FP8_E4M3 = 2, SPARK_INT8 = 3 } spark_dtype;

/* What StatTop_k writes for entries at or below theta: 0 (Eq.10) or -inf (the Top_k^(-inf)
 * variant used in front of a softmax, Section 3 after Eq.11). */
typedef enum { SPARK_FILL_ZERO = 0, SPARK_FILL_NEG_INF = 1 } spark_fill;

/* GELU form: exact x*Phi(x) (default) or its tanh approximation. */
typedef enum { SPARK_GELU_ERF = 0, SPARK_GELU_TANH = 1 } spark_gelu;

/* Host. Static string for a status code. */
const char* spark_status_string(spark_status s);

/* Host. Library version (SPARK_VERSION it was built with). */
int spark_version(void);

/* Host. Q(p): quantile of the standard Gaussian (Section 3, text after Eq.11), accurate to
 * a few ulp in double.  Q(0) = -inf, Q(1) = +inf, NaN outside [0, 1]. */
double spark_normal_quantile(double p);

/* ------------------------------------------------------------------------------------------
 * Row-wise statistical top-k (Eq.9-11), the operator applied to the [tokens x d_ff]
 * pre-activation tensor in training / prefill and to the predictor scores in decode.
 *
 *   x      [rows][n] of `dt`, row pitch ldx elements (ldx >= n)                    in
 *   k      target number of survivors per row, 1 <= k <= n-1
 *   y      [rows][n] of `dt`, row pitch ldy; y = x - theta where x > theta,        out, optional
 *          else the fill value.  Computed in fp32, rounded to nearest-even on
 *          store for bf16.  May alias x exactly (in place).
 *   theta  [rows] fp32 threshold of each row                                       out, optional
 *   count  [rows] int32, #{i : x_i > theta} (strict), exact even if idx is capped  out, optional
 *   idx    [rows][idx_cap] int32, ascending active indices; entries past           out, optional
 *          min(count, idx_cap) are left untouched
 *
 * Statistics are accumulated in fp32 (mean first, then centred squares) whatever `dt` is.
 * A constant row has std = 0, theta = mean and no survivor.  n >= 2 is required.
 * Needs no workspace.  Errors: NULL x; rows < 0, n < 2, n > 2^31-1 or a pitch < n -> SHAPE;
 * k out of range -> K; dt -> DTYPE; alignment -> ALIGN.
 */
/* Host. Bytes of device workspace spark_stat_topk needs: always 0 (a row stays on chip between
 * its statistics and its thresholding). */
size_t spark_stat_topk_workspace_bytes(int64_t rows, int64_t n);

spark_status spark_stat_topk(const void* x, spark_dtype dt, int64_t rows, int64_t n, int64_t ldx,
                             int64_t k, spark_fill fill, void* y, int64_t ldy, float* theta,
                             int32_t* count, int32_t* idx, int64_t idx_cap, void* hip_stream);

/*
 * Statistical top-k of rows whose columns are sharded over several devices (Appendix D.2, the
 * global variant: every device contributes the statistics of its shard, the combined
 * statistics give one threshold per row, and each device thresholds its own shard with it; the
 * result is that of the unsharded operator).  One device's share, in three calls; the exchange of
 * the statistics between the devices (8 bytes per row and shard) is the caller's.  The local
 * variant of the same appendix (k / m on every shard, no exchange, a different result) is
 * spark_stat_topk applied to the shard with k' = k / m.
 *
 * spark_stat_topk_shard_stats: the statistics of this device's shard.
 *   x      [rows][n_shard] of `dt`, row pitch ldx elements (>= n_shard), device, 16-byte aligned
 *   stats  [rows][2] fp32, device: mean and centred sum of squares sum (x - mean)^2 of each row  out
 * spark_stat_topk_combine_stats: thresholds from the statistics of all shards, combined in shard
 * order (mean = sum n_s mean_s / N, M2 = sum (M2_s + n_s (mean_s - mean)^2)):
 *   stats    [n_shards][rows][2] fp32, device (the arrays the shards produced, gathered)
 *   n_shard  [n_shards] entries per shard, HOST array; 1 <= n_shards <= SPARK_MAX_SHARDS,
 *            N = sum n_shard >= 2
 *   k        1 <= k <= N - 1 (the sparsity level of the whole rows)
 *   theta    [rows] fp32, device: mean + std Q(1 - k / N), std with divisor N - 1 (Eq.11)  out
 *   mean, std [rows] fp32, device                                                out, optional
 * spark_stat_topk_apply: soft thresholding of this device's shard with the given thresholds:
 *   y = x - theta where x > theta, the fill value elsewhere; count / idx as in spark_stat_topk
 *   (indices inside the shard).  y may alias x exactly.
 *
 * Errors as spark_stat_topk (n_shard >= 1 here).  No workspace; asynchronous on hip_stream.
 */
#define SPARK_MAX_SHARDS 64
spark_status spark_stat_topk_shard_stats(const void* x, spark_dtype dt, int64_t rows, int64_t n_shard,
                                         int64_t ldx, float* stats, void* hip_stream);
spark_status spark_stat_topk_combine_stats(const float* stats, const int64_t* n_shard, int32_t n_shards,
                                           int64_t rows, int64_t k, float* theta, float* mean,
                                           float* std, void* hip_stream);
spark_status spark_stat_topk_apply(const void* x, spark_dtype dt, int64_t rows, int64_t n_shard,
                                   int64_t ldx, const float* theta, spark_fill fill, void* y,
                                   int64_t ldy, int32_t* count, int32_t* idx, int64_t idx_cap,
                                   void* hip_stream);

/*
 * The continuously differentiable variant of Section 3.2 (Eq.13, Eq.14, Theorem 2):
 *   y = Huber(StatTop_k(x); delta) / delta,  Huber(a; delta) = a^2 / 2 for |a| < delta,
 *                                            delta (|a| - delta / 2) otherwise,
 * row by row; delta = 0 is the limit the paper uses in practice, y = StatTop_k(x).
 *
 *   x, y   [rows][n] of `dt`, row pitches ldx, ldy elements (>= n); y may alias x exactly
 *   delta  >= 0, finite
 *   theta  [rows] fp32                                                            out, optional
 *
 * fp32 arithmetic, rounded to nearest-even on store for bf16.  Needs no workspace.
 * Errors as spark_stat_topk; delta negative, NaN or infinite -> SHAPE.
 */
spark_status spark_stat_topk_huber(const void* x, spark_dtype dt, int64_t rows, int64_t n,
                                   int64_t ldx, int64_t k, float delta, void* y, int64_t ldy,
                                   float* theta, void* hip_stream);

/*
 * Backward pass of spark_stat_topk_huber (and, with delta = 0, of spark_stat_topk with zero
 * fill): gx[row] = gy[row] . dy/dx.  The gradient flows through the threshold as well
 * (theta is a linear combination of the row's mean and standard deviation, both functions of
 * x: Appendix A.2):
 *   w_i  = gy_i * h'(x_i - theta) where x_i > theta, else 0,  h'(a) = a / delta below delta, else 1
 *   gx_j = w_j - (sum_i w_i) * (1/n + Q(1 - k/n) (x_j - mean) / ((n - 1) std)).
 * With delta = 0 the operator is not differentiable where an entry equals theta; the
 * one-sided value 0 is used there.  A constant row (std = 0) keeps nothing and gets gx = 0.
 *
 *   x, gy, gx  [rows][n] of `dt`, row pitches ldx, ldgy, ldgx; gx may alias gy or x exactly
 *
 * Each of x and gy is read once and gx written once (rows up to 24576 fp32 / 32768 bf16
 * elements; longer rows are re-read).  fp32 arithmetic.  Needs no workspace.  Errors as above.
 */
spark_status spark_stat_topk_huber_backward(const void* x, const void* gy, spark_dtype dt,
                                            int64_t rows, int64_t n, int64_t ldx, int64_t ldgy,
                                            int64_t k, float delta, void* gx, int64_t ldgx,
                                            void* hip_stream);

/* ------------------------------------------------------------------------------------------
 * One Spark-FFN layer (Eq.2).  Host struct holding device pointers.
 */
/* 8-bit weights (wdtype = SPARK_FP8_E4M3 or SPARK_INT8; the quantisation synergy of Appendix D.4: the sparse
 * path touches half the bytes again).  Each of the three arrays is then one allocation holding
 * the codes [d_ff][cols], one byte each, immediately followed by d_ff fp32 scales, one per
 * row: weight[j][c] = scale[j] * value(code[j][c]).  cols (r, d_model - r, d_model) must be
 * multiples of 16.  One token per call (spark_ffn_decode, spark_ffn_decode_layers,
 * spark_ffn_dense_decode_layers, spark_ffn_prefill with chunk 1) takes the bandwidth-bound
 * phase-by-phase kernels; 2 to 64 bf16 tokens (and prefill chunks of that size) with r and
 * d_model - r multiples of 256 (1024, 1280, 1536 or 2048 for at most 16 tokens; 512 to 1536 above
 * that, and 2048 for at most 32) take the batched matrix-core kernels, which widen the codes to
 * bf16 (exact for both kinds); every other batch is evaluated by the general kernels (a launch sequence per layer,
 * not tuned); the dense comparison calls take one token only
 * (SPARK_ERR_DTYPE otherwise).  Arithmetic: codes widened exactly, fp32 products and sums, the
 * row's scale applied to the finished dot product. */
typedef struct {
  int32_t d_model;    /* input / output width                                   */
  int32_t d_ff;       /* number of neurons, >= 2                                */
  int32_t r;          /* predictor width, 1 <= r <= d_model-1                   */
  int32_t k;          /* sparsity level, 1 <= k <= d_ff-1                       */
  int32_t wdtype;     /* spark_dtype of the three weight arrays                 */
  int32_t gelu;       /* spark_gelu                                             */
  const void* k1n;    /* [d_ff][r]            predictor half of the first layer */
  const void* k2n;    /* [d_ff][d_model - r]  gated half of the first layer     */
  const void* vn;     /* [d_ff][d_model]      second layer                      */
} spark_ffn_layer;

/* Host. Bytes of device workspace spark_ffn_decode / spark_ffn_decode_layers /
 * spark_ffn_dense_decode need for this layer shape and batch (0 on invalid arguments). */
size_t spark_ffn_workspace_bytes(int32_t d_model, int32_t d_ff, int32_t batch);

/*
 * Decode `batch` tokens through one layer (Section 2.1; batching as in Appendix B: each
 * token has its own threshold and mask, the union of the masks decides which weight rows
 * are fetched, and y[b] does not depend on the other tokens of the batch).
 *
 *   q             [batch][d_model] of `qdtype`, row pitch ldq elements             in
 *   y             [batch][d_model] fp32, overwritten                               out
 *   theta         [batch] fp32                                                     out, optional
 *   active_count  [batch] int32, #{j : s_bj > theta_b}                             out, optional
 *   active_idx    [batch][d_ff] int32, ascending active neurons of each token      out, optional
 *   union_count   [1] int32, size of the union of the active sets                  out, optional
 *   union_idx     [d_ff] int32, ascending union                                    out, optional
 *   workspace     >= spark_ffn_workspace_bytes(d_model, d_ff, batch), 256-byte aligned
 *
 * Arithmetic: weights and q are widened exactly to fp32; all products and sums are fp32
 * (bf16 x bf16 products are exact in fp32); q is never rounded by the library.
 * 1 <= batch <= SPARK_MAX_BATCH.
 */
spark_status spark_ffn_decode(const spark_ffn_layer* layer, const void* q, spark_dtype qdtype,
                              int32_t batch, int64_t ldq, float* y, float* theta,
                              int32_t* active_count, int32_t* active_idx, int32_t* union_count,
                              int32_t* union_idx, void* workspace, size_t workspace_bytes,
                              void* hip_stream);

/*
 * spark_ffn_decode for callers that can neither allocate device memory nor pass a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments
 * (minus the workspace), same kernels and same results as spark_ffn_decode for one token; the
 * scratch memory is an array of SPARK_STATIC_SCRATCH_BYTES built into the library's code object
 * (every GPU the library runs on holds its copy until the process ends).  The call allocates and
 * frees nothing; the first call on a device looks up the array's address on that device (make it
 * outside a stream capture).
 *
 * Limits: batch = 1 and a shape the one-token kernels take (rows of at most 256 16-byte chunks
 * for K1n, 448 for Vn with bf16 weights; others -> SPARK_ERR_SHAPE), and a scratch need of
 * 4 d_ff + 8 ceil(d_ff / 16) + 256 d_model bytes (each term rounded up to 256) within
 * SPARK_STATIC_SCRATCH_BYTES (-> SPARK_ERR_WORKSPACE beyond; the 2B and 9B layer shapes need 0.6
 * and 1.0 MB).  Other errors as spark_ffn_decode.
 *
 * All calls on one GPU share that GPU's array: calls that may overlap in time (different streams,
 * different threads) race on it and must be ordered by the caller.  Nothing in the array has to
 * start at zero, and a call leaves nothing behind that a later call depends on.
 */
#define SPARK_STATIC_SCRATCH_BYTES (2u << 20)
spark_status spark_ffn_decode_static(const spark_ffn_layer* layer, const void* q, spark_dtype qdtype,
                                     int32_t batch, int64_t ldq, float* y, float* theta,
                                     int32_t* active_count, int32_t* active_idx, int32_t* union_count,
                                     int32_t* union_idx, void* hip_stream);

/*
 * n_layers independent layers of one shape, evaluated in order l = 0 .. n_layers-1 on the
 * same q (host array `layers`; every layer must agree in d_model, d_ff, r, k, wdtype, gelu).
 * Output arrays carry a leading n_layers dimension:
 *   y [n_layers][batch][d_model], theta [n_layers][batch], active_count [n_layers][batch],
 *   active_idx [n_layers][batch][d_ff], union_count [n_layers], union_idx [n_layers][d_ff].
 * The layers are independent (they share q), so every step of the path - predictor sweep,
 * thresholds and compaction, gathered products, final sums - is one launch over all layers;
 * results are the same as n_layers calls of spark_ffn_decode.
 */
spark_status spark_ffn_decode_layers(const spark_ffn_layer* layers, int32_t n_layers,
                                     const void* q, spark_dtype qdtype, int32_t batch,
                                     int64_t ldq, float* y, float* theta, int32_t* active_count,
                                     int32_t* active_idx, int32_t* union_count,
                                     int32_t* union_idx, void* workspace,
                                     size_t workspace_bytes, void* hip_stream);

/* Host. Bytes of device workspace spark_ffn_prefill needs for this layer shape and chunk size
 * (0 on invalid arguments). */
size_t spark_ffn_prefill_workspace_bytes(int32_t d_model, int32_t d_ff, int32_t chunk);

/*
 * Prefill: n_tokens tokens of a prompt through one layer, in chunks of `chunk` consecutive
 * tokens (Section 4.3 and Appendix B: the prompt is processed in chunks, 64 tokens in the
 * paper's set-up; within a chunk every token keeps its own threshold and mask, and the
 * union of the chunk's masks decides which weight rows are fetched).  Token t belongs to
 * chunk t / chunk; the last chunk may be shorter.  Every y[t] equals what spark_ffn_decode
 * gives for that token alone.
 *
 *   q             [n_tokens][d_model] of `qdtype`, row pitch ldq elements          in
 *   y             [n_tokens][d_model] fp32, overwritten                            out
 *   theta         [n_tokens] fp32                                                  out, optional
 *   active_count  [n_tokens] int32                                                 out, optional
 *   active_idx    [n_tokens][d_ff] int32, ascending active neurons of each token   out, optional
 *   union_count   [ceil(n_tokens / chunk)] int32, union size of each chunk         out, optional
 *   union_idx     [ceil(n_tokens / chunk)][d_ff] int32, ascending union per chunk  out, optional
 *   workspace     >= spark_ffn_prefill_workspace_bytes(d_model, d_ff, chunk), 256-byte aligned
 *
 * 1 <= chunk <= SPARK_MAX_BATCH; n_tokens = 0 is a no-op.  The full chunks are independent
 * and are evaluated step by step over all chunks at once (bf16 weights and tokens; other
 * types chunk by chunk).  Arithmetic and errors as for spark_ffn_decode.
 */
spark_status spark_ffn_prefill(const spark_ffn_layer* layer, const void* q, spark_dtype qdtype,
                               int64_t n_tokens, int32_t chunk, int64_t ldq, float* y,
                               float* theta, int32_t* active_count, int32_t* active_idx,
                               int32_t* union_count, int32_t* union_idx, void* workspace,
                               size_t workspace_bytes, void* hip_stream);

/*
 * Dense evaluation of the same layer (every neuron's K2 and V row is read; the result
 * equals spark_ffn_decode's because inactive neurons contribute exact zeros).  It exists as
 * the same-GPU comparison point for the sparse path (Eq.3 vs Eq.4).
 */
spark_status spark_ffn_dense_decode(const spark_ffn_layer* layer, const void* q,
                                    spark_dtype qdtype, int32_t batch, int64_t ldq, float* y,
                                    void* workspace, size_t workspace_bytes, void* hip_stream);

/* The same for n_layers independent layers on the same q (y [n_layers][batch][d_model]); for
 * batch 1 the layers are evaluated phase by phase over the whole stack like
 * spark_ffn_decode_layers, with every K2 / V row fetched. */
spark_status spark_ffn_dense_decode_layers(const spark_ffn_layer* layers, int32_t n_layers,
                                           const void* q, spark_dtype qdtype, int32_t batch,
                                           int64_t ldq, float* y, void* workspace,
                                           size_t workspace_bytes, void* hip_stream);

/* ------------------------------------------------------------------------------------------
 * Spark-attention decode (Section 2.2, Eq.7): for every query head,
 *   y = V ( softmax( Top_k^(-inf)( K1^T q[:r] ) ) * softplus( K2^T q[r:] ) ),
 * Top_k^(-inf) being the statistical top-k of Eq.9-11 that sets the entries at or below the
 * threshold to -inf (text after Eq.11).  One cache serves `group` query heads.
 * Host struct holding device pointers; the caches are token-major:
 */
typedef struct {
  int32_t n_ctx;      /* cached keys, 1 .. 16384                                   */
  int32_t d_attn;     /* head width                                                */
  int32_t r;          /* predictor width, 1 <= r <= d_attn-1                       */
  int32_t k;          /* keys to keep, >= 1; n_ctx <= k keeps every key            */
  int32_t cdtype;     /* spark_dtype of the three caches                           */
  int32_t group;      /* query heads sharing this cache, 1 .. 4                    */
  const void* k1c;    /* [n_ctx][r]           first r entries of every key         */
  const void* k2c;    /* [n_ctx][d_attn - r]  the rest of every key                */
  const void* vc;     /* [n_ctx][d_attn]      values                               */
} spark_attn_head;

/* Host. Bytes of device workspace spark_attn_decode needs (0 on invalid arguments). */
size_t spark_attn_workspace_bytes(int32_t n_heads, int32_t group, int32_t n_ctx);

/*
 * One decode step of n_heads caches (host array `heads`; all must agree in n_ctx, d_attn, r,
 * k, cdtype, group), one query per query head.
 *
 *   q           [n_heads][group][d_attn] of `qdtype`, contiguous                    in
 *   y           [n_heads][group][d_attn] fp32, overwritten                          out
 *   theta       [n_heads][group] fp32 (-inf when n_ctx <= k)                        out, optional
 *   kept_count  [n_heads][group] int32, #{i : s_i > theta}                          out, optional
 *   kept_idx    [n_heads][group][n_ctx] int32, ascending kept keys; entries past    out, optional
 *               the count are left untouched
 *   workspace   >= spark_attn_workspace_bytes(n_heads, group, n_ctx), 256-byte aligned
 *
 * Arithmetic: caches and q widened exactly to fp32, products and sums fp32; the softmax is
 * evaluated as exp(s - max s) over the kept keys divided by its sum.  No 1/sqrt(d) factor is
 * applied (Eq.7 carries none: fold it into q).  If no score exceeds theta (all scores equal)
 * y = 0.  Supported shapes: r, d_attn - r and d_attn each a power-of-two number of 16-byte
 * chunks (4..64 for r, 4..32 for d_attn - r, 8..64 for d_attn); others -> SHAPE.
 */
spark_status spark_attn_decode(const spark_attn_head* heads, int32_t n_heads, const void* q,
                               spark_dtype qdtype, float* y, float* theta, int32_t* kept_count,
                               int32_t* kept_idx, void* workspace, size_t workspace_bytes,
                               void* hip_stream);

/* ------------------------------------------------------------------------------------------
 * Testing and measurement aids.
 */

/* Host struct.  Choices a caller may pin for one spark_ffn_decode_layers_tuned call instead of
 * leaving them to the library; every field 0 = automatic.  Results do not depend on them beyond
 * the order of fp32 additions. */
typedef struct {
  int32_t path;                     /* 1 = the general multi-kernel path even where a phase-by-phase
                                       path exists (8-bit weights have no general path: ignored)    */
  int32_t phases;                   /* one-token path: which launches the call makes: bit 0 the
                                       predictor sweep, bit 1 the gather, bit 2 the reduction (and the
                                       index lists).  A call that skips a launch finds that launch's
                                       outputs as an earlier full call on the same workspace left
                                       them, so each kernel can be timed alone on valid inputs       */
  int32_t rows_per_predict_block;   /* one token: rows per workgroup of the predictor sweep; batches:
                                       16 x the tiles per workgroup of the predict step              */
  int32_t neurons_per_gather_block; /* one token: neurons per workgroup of the gather; batches: 16 x
                                       the tiles per workgroup of the k2 step                        */
  int32_t variant;                  /* one token: 1 = the 8-wave gather variant; batches: 100 x kernel
                                       family + row slices of the V step, families 1 = k-split kernels
                                       for every batch size, 4 = whole-row kernels wherever they are
                                       compiled, 5 = LDS-staged kernels wherever they are compiled   */
} spark_ffn_tuning;

/* spark_ffn_decode_layers with pinned choices (`tuning` is a host pointer, NULL = automatic). */
spark_status spark_ffn_decode_layers_tuned(const spark_ffn_layer* layers, int32_t n_layers,
                                           const void* q, spark_dtype qdtype, int32_t batch,
                                           int64_t ldq, float* y, float* theta, int32_t* active_count,
                                           int32_t* active_idx, int32_t* union_count,
                                           int32_t* union_idx, void* workspace,
                                           size_t workspace_bytes, const spark_ffn_tuning* tuning,
                                           void* hip_stream);

/* A plain device-to-device copy kernel (dst, src 16-byte aligned, nbytes a multiple of 16; the
 * ranges must not overlap): it reads exactly nbytes and writes exactly nbytes, which makes it the
 * known-size reference the HBM byte counters are scaled by when kernel traffic is measured. */
spark_status spark_copy_bytes(void* dst, const void* src, size_t nbytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SPARK_H_ */
