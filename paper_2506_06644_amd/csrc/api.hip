// C ABI of the Spark-FFN library: host-side validation and dispatch.  See include/spark.h.
#include "../../include/spark.h"

#include <atomic>
#include <cmath>
#include <limits>

#include "spark_internal.h"

// Scratch memory of spark_ffn_decode_static: one copy per GPU, held until the process ends.
static __device__ __align__(256) unsigned char scratch[SPARK_STATIC_SCRATCH_BYTES];

namespace {

// Device address of `scratch` on the current device, looked up once per device (every GPU holds
// its own copy of the array at its own address; in host code the array's name is not an address).
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

hipError_t static_scratch_address(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!ptr) {
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);  // two threads racing here store the same address
  }
  *out = ptr;
  return hipSuccess;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool is_code_dtype(int dt) { return dt == SPARK_FP8_E4M3 || dt == SPARK_INT8; }  // 8-bit codes with row scales
size_t dtype_size(int dt) { return is_code_dtype(dt) ? 1 : dt == SPARK_BF16 ? 2 : 4; }
bool dtype_ok(int dt) { return dt == SPARK_F32 || dt == SPARK_BF16; }            // tokens, activations
bool weight_dtype_ok(int dt) { return dtype_ok(dt) || is_code_dtype(dt); }  // weight arrays

double normal_cdf(double z) { return 0.5 * std::erfc(-z * 0.70710678118654752440); }

spark_status validate_layer(const spark_ffn_layer* L) {
  if (!L) return SPARK_ERR_NULL;
  if (!L->k1n || !L->k2n || !L->vn) return SPARK_ERR_NULL;
  if (!weight_dtype_ok(L->wdtype)) return SPARK_ERR_DTYPE;
  if (L->gelu != SPARK_GELU_ERF && L->gelu != SPARK_GELU_TANH) return SPARK_ERR_DTYPE;
  if (L->d_ff < 2 || L->d_model < 2) return SPARK_ERR_SHAPE;
  if (L->r < 1 || L->r > L->d_model - 1) return SPARK_ERR_SHAPE;
  if (L->k < 1 || L->k > L->d_ff - 1) return SPARK_ERR_K;
  const size_t ws = dtype_size(L->wdtype);
  if ((L->r * ws) % 16 || ((L->d_model - L->r) * ws) % 16 || (L->d_model * ws) % 16) return SPARK_ERR_ALIGN;
  if (!aligned16(L->k1n) || !aligned16(L->k2n) || !aligned16(L->vn)) return SPARK_ERR_ALIGN;
  return SPARK_OK;
}

spark::FfnProblem make_problem(const spark_ffn_layer* L, const void* q, int qdtype, int32_t batch, int64_t ldq,
                               float* y, float* theta, int32_t* active_count, int32_t* active_idx,
                               int32_t* union_count, int32_t* union_idx);

// Everything about a decode call but its workspace.
spark_status validate_decode_args(const spark_ffn_layer* L, const void* q, int qdtype, int32_t batch, int64_t ldq,
                                  const float* y) {
  spark_status s = validate_layer(L);
  if (s != SPARK_OK) return s;
  if (!q || !y) return SPARK_ERR_NULL;
  if (!dtype_ok(qdtype)) return SPARK_ERR_DTYPE;
  if (batch < 1 || batch > SPARK_MAX_BATCH) return SPARK_ERR_SHAPE;
  if (ldq < L->d_model) return SPARK_ERR_SHAPE;
  const size_t qs = dtype_size(qdtype);
  // the split point r and every token row must fall on a 16-byte boundary of q as well
  if (!aligned16(q) || (ldq * qs) % 16 || (L->r * qs) % 16 || (L->d_model * qs) % 16) return SPARK_ERR_ALIGN;
  return SPARK_OK;
}

spark_status validate_decode(const spark_ffn_layer* L, const void* q, int qdtype, int32_t batch, int64_t ldq,
                             const float* y, const void* workspace, size_t workspace_bytes) {
  const spark_status s = validate_decode_args(L, q, qdtype, batch, ldq, y);
  if (s != SPARK_OK) return s;
  if (!workspace) return SPARK_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return SPARK_ERR_WORKSPACE;
  if (workspace_bytes < spark_ffn_workspace_bytes(L->d_model, L->d_ff, batch)) return SPARK_ERR_WORKSPACE;
  if (is_code_dtype(L->wdtype) && batch == 1) {
    // one token with 8-bit weights: the phase-by-phase kernels only (batches take the general kernels)
    const spark::FfnProblem p = make_problem(L, q, qdtype, batch, ldq, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr);
    if (!spark::phased_supported(p)) return SPARK_ERR_DTYPE;
  }
  return SPARK_OK;
}

spark::FfnProblem make_problem(const spark_ffn_layer* L, const void* q, int qdtype, int32_t batch, int64_t ldq,
                               float* y, float* theta, int32_t* active_count, int32_t* active_idx,
                               int32_t* union_count, int32_t* union_idx) {
  spark::FfnProblem p;
  p.d_model = L->d_model;
  p.d_ff = L->d_ff;
  p.r = L->r;
  p.k = L->k;
  p.w_bf16 = L->wdtype == SPARK_BF16;
  p.w_fp8 = L->wdtype == SPARK_FP8_E4M3 ? 1 : L->wdtype == SPARK_INT8 ? 2 : 0;
  p.q_bf16 = qdtype == SPARK_BF16;
  p.gelu = L->gelu;
  p.k1n = L->k1n;
  p.k2n = L->k2n;
  p.vn = L->vn;
  p.q = q;
  p.ldq = ldq;
  p.batch = batch;
  p.z = (float)spark_normal_quantile(1.0 - (double)L->k / (double)L->d_ff);
  p.y = y;
  p.theta = theta;
  p.active_count = active_count;
  p.active_idx = active_idx;
  p.union_count = union_count;
  p.union_idx = union_idx;
  return p;
}

// partial output rows the phase-by-phase region of a caller's workspace holds (64 per layer of a set of launches)
constexpr int kWorkspacePartRows = spark::kPhasedMaxLayers * 64;

spark::FfnTuning make_tuning(const spark_ffn_tuning* t) {
  spark::FfnTuning u;
  if (t) {
    u.path = t->path == 1 ? 1 : 0;
    u.phases = t->phases;
    u.rows_per_predict_block = t->rows_per_predict_block;
    u.neurons_per_gather_block = t->neurons_per_gather_block;
    u.variant = t->variant;
  }
  return u;
}

// May this problem take a phase-by-phase path under this tuning?  (8-bit weights have no other.)
bool takes_phased(const spark::FfnProblem& p, const spark::FfnTuning& tune) {
  return (tune.path == 0 || p.w_fp8) && (spark::phased_supported(p) || spark::phased_batch_supported(p));
}

// Runs layers[0..n) phase by phase: the one-token path or the batched path on the matrix cores.
// `scratch` is laid out for `layer_cap` layers per set of launches (one-token path).
hipError_t run_phased(const spark_ffn_layer* layers, int32_t n_layers, const spark::FfnProblem& p0,
                      const spark::FfnTuning& tune, void* scratch, int layer_cap, int part_rows, hipStream_t st,
                      int dense = 0) {
  const void* k1n[256];
  const void* k2n[256];
  const void* vn[256];
  hipError_t e = hipSuccess;
  for (int32_t base = 0; base < n_layers && e == hipSuccess; base += 256) {
    const int32_t n = n_layers - base < 256 ? n_layers - base : 256;
    for (int32_t l = 0; l < n; ++l) {
      k1n[l] = layers[base + l].k1n;
      k2n[l] = layers[base + l].k2n;
      vn[l] = layers[base + l].vn;
    }
    spark::FfnProblem p = p0;
    p.y = p0.y + (int64_t)base * p0.batch * p0.d_model;
    if (p.theta) p.theta += (int64_t)base * p0.batch;
    if (p.active_count) p.active_count += (int64_t)base * p0.batch;
    if (p.active_idx) p.active_idx += (int64_t)base * p0.batch * p0.d_ff;
    if (p.union_count) p.union_count += base;
    if (p.union_idx) p.union_idx += (int64_t)base * p0.d_ff;
    if (p.batch >= 2) e = spark::launch_ffn_phased_batch(p, k1n, k2n, vn, n, tune, scratch, st);
    else e = spark::launch_ffn_phased(p, k1n, k2n, vn, n, dense, tune, scratch, layer_cap, part_rows, st);
  }
  return e;
}

spark_status decode_layers(const spark_ffn_layer* layers, int32_t n_layers, const void* q, spark_dtype qdtype,
                           int32_t batch, int64_t ldq, float* y, float* theta, int32_t* active_count,
                           int32_t* active_idx, int32_t* union_count, int32_t* union_idx, void* workspace,
                           size_t workspace_bytes, const spark::FfnTuning& tune, hipStream_t st) {
  if (!layers) return SPARK_ERR_NULL;
  if (n_layers < 1) return SPARK_ERR_SHAPE;
  for (int32_t l = 0; l < n_layers; ++l) {
    const spark_status s = validate_decode(&layers[l], q, qdtype, batch, ldq, y, workspace, workspace_bytes);
    if (s != SPARK_OK) return s;
    if (layers[l].d_model != layers[0].d_model || layers[l].d_ff != layers[0].d_ff ||
        layers[l].r != layers[0].r || layers[l].k != layers[0].k || layers[l].wdtype != layers[0].wdtype ||
        layers[l].gelu != layers[0].gelu)
      return SPARK_ERR_SHAPE;
  }
  const int64_t d_model = layers[0].d_model, d_ff = layers[0].d_ff;
  const spark::FfnWorkspace ws = spark::carve_workspace(workspace, layers[0].d_model, layers[0].d_ff, batch);
  const spark::FfnProblem p0 = make_problem(&layers[0], q, qdtype, batch, ldq, y, theta, active_count, active_idx,
                                            union_count, union_idx);
  if (takes_phased(p0, tune)) {
    const hipError_t e = run_phased(layers, n_layers, p0, tune, ws.phased, spark::kPhasedMaxLayers, kWorkspacePartRows, st);
    return e == hipSuccess ? SPARK_OK : SPARK_ERR_DEVICE;
  }
  for (int32_t l = 0; l < n_layers; ++l) {
    const spark::FfnProblem p = make_problem(
        &layers[l], q, qdtype, batch, ldq, y + (int64_t)l * batch * d_model,
        theta ? theta + (int64_t)l * batch : nullptr, active_count ? active_count + (int64_t)l * batch : nullptr,
        active_idx ? active_idx + (int64_t)l * batch * d_ff : nullptr, union_count ? union_count + l : nullptr,
        union_idx ? union_idx + (int64_t)l * d_ff : nullptr);
    if (spark::launch_ffn_general(p, ws, 0, st) != hipSuccess) return SPARK_ERR_DEVICE;
  }
  return SPARK_OK;
}

}  // namespace

extern "C" {

const char* spark_status_string(spark_status s) {
  switch (s) {
    case SPARK_OK: return "ok";
    case SPARK_ERR_NULL: return "required pointer is null";
    case SPARK_ERR_SHAPE: return "dimension, stride or batch out of range";
    case SPARK_ERR_K: return "k outside [1, d-1]";
    case SPARK_ERR_DTYPE: return "unsupported dtype or activation kind";
    case SPARK_ERR_ALIGN: return "pointer or row pitch not 16-byte aligned";
    case SPARK_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case SPARK_ERR_DEVICE: return "HIP runtime error";
  }
  return "unknown status";
}

int spark_version(void) { return SPARK_VERSION; }

// Q(p) by a rational starting guess for the tail (Hastings' approximation, A&S 26.2.23)
// polished with Halley steps on Phi(z) - p, where Phi is evaluated through erfc so the lower
// tail keeps its relative accuracy.
double spark_normal_quantile(double p) {
  if (std::isnan(p) || p < 0.0 || p > 1.0) return std::numeric_limits<double>::quiet_NaN();
  if (p == 0.0) return -std::numeric_limits<double>::infinity();
  if (p == 1.0) return std::numeric_limits<double>::infinity();
  if (p == 0.5) return 0.0;
  const bool upper = p > 0.5;
  const double pl = upper ? 1.0 - p : p;  // lower-tail mass, in (0, 1/2)
  const double t = std::sqrt(-2.0 * std::log(pl));
  double z = -(t - (2.515517 + t * (0.802853 + t * 0.010328)) /
                       (1.0 + t * (1.432788 + t * (0.189269 + t * 0.001308))));
  const double inv_sqrt_2pi = 0.39894228040143267794;
  for (int it = 0; it < 8; ++it) {
    const double f = normal_cdf(z) - pl;
    const double pdf = inv_sqrt_2pi * std::exp(-0.5 * z * z);
    if (pdf == 0.0) break;
    const double u = f / pdf;
    const double step = u / (1.0 + 0.5 * z * u);
    z -= step;
    if (std::fabs(step) <= 1e-16 * std::fabs(z)) break;
  }
  return upper ? -z : z;
}

spark_status spark_stat_topk(const void* x, spark_dtype dt, int64_t rows, int64_t n, int64_t ldx, int64_t k,
                             spark_fill fill, void* y, int64_t ldy, float* theta, int32_t* count,
                             int32_t* idx, int64_t idx_cap, void* hip_stream) {
  if (!x) return SPARK_ERR_NULL;
  if (!dtype_ok(dt)) return SPARK_ERR_DTYPE;
  if (fill != SPARK_FILL_ZERO && fill != SPARK_FILL_NEG_INF) return SPARK_ERR_DTYPE;
  if (rows < 0 || rows > 2147483647LL || n < 2 || n > 2147483647LL || ldx < n) return SPARK_ERR_SHAPE;
  if (y && ldy < n) return SPARK_ERR_SHAPE;
  if (idx && idx_cap < 0) return SPARK_ERR_SHAPE;
  if (k < 1 || k > n - 1) return SPARK_ERR_K;
  const size_t es = dtype_size(dt);
  if (!aligned16(x) || (ldx * es) % 16) return SPARK_ERR_ALIGN;
  if (y && (!aligned16(y) || (ldy * es) % 16)) return SPARK_ERR_ALIGN;
  const float z = (float)spark_normal_quantile(1.0 - (double)k / (double)n);
  const hipError_t e = spark::launch_stat_topk(x, dt == SPARK_BF16, rows, n, ldx, z, fill == SPARK_FILL_NEG_INF, 0.f,
                                               y, ldy, theta, count, idx, idx_cap, nullptr,
                                               static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? SPARK_OK : SPARK_ERR_DEVICE;
}

spark_status spark_stat_topk_shard_stats(const void* x, spark_dtype dt, int64_t rows, int64_t n_shard, int64_t ldx,
                                         float* stats, void* hip_stream) {
  if (!x || !stats) return SPARK_ERR_NULL;
  if (!dtype_ok(dt)) return SPARK_ERR_DTYPE;
  if (rows < 0 || rows > 2147483647LL || n_shard < 1 || n_shard > 2147483647LL || ldx < n_shard) return SPARK_ERR_SHAPE;
  const size_t es = dtype_size(dt);
  if (!aligned16(x) || (ldx * es) % 16) return SPARK_ERR_ALIGN;
  const hipError_t e = spark::launch_stat_topk(x, dt == SPARK_BF16, rows, n_shard, ldx, 0.f, 0, 0.f, nullptr, 0, nullptr,
                                               nullptr, nullptr, 0, nullptr, static_cast<hipStream_t>(hip_stream), nullptr,
                                               stats);
  return e == hipSuccess ? SPARK_OK : SPARK_ERR_DEVICE;
}

spark_status spark_stat_topk_combine_stats(const float* stats, const int64_t* n_shard, int32_t n_shards, int64_t rows,
                                           int64_t k, float* theta, float* mean, float* std, void* hip_stream) {
  if (!stats || !n_shard || !theta) return SPARK_ERR_NULL;
  if (rows < 0 || rows > 2147483647LL || n_shards < 1 || n_shards > SPARK_MAX_SHARDS) return SPARK_ERR_SHAPE;
  int64_t total = 0;
  for (int32_t s = 0; s < n_shards; ++s) {
    if (n_shard[s] < 1 || n_shard[s] > 2147483647LL) return SPARK_ERR_SHAPE;
    total += n_shard[s];
  }
  if (total < 2 || total > 2147483647LL) return SPARK_ERR_SHAPE;
  if (k < 1 || k > total - 1) return SPARK_ERR_K;
  const float z = (float)spark_normal_quantile(1.0 - (double)k / (double)total);
  const hipError_t e = spark::launch_combine_shard_stats(stats, n_shard, n_shards, rows, z, theta, mean, std,
                                                         static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? SPARK_OK : SPARK_ERR_DEVICE;
}

spark_status spark_stat_topk_apply(const void* x, spark_dtype dt, int64_t rows, int64_t n_shard, int64_t ldx,
                                   const float* theta, spark_fill fill, void* y, int64_t ldy, int32_t* count,
                                   int32_t* idx, int64_t idx_cap, void* hip_stream) {
  if (!x || !theta) return SPARK_ERR_NULL;
  if (!dtype_ok(dt)) return SPARK_ERR_DTYPE;
  if (fill != SPARK_FILL_ZERO && fill != SPARK_FILL_NEG_INF) return SPARK_ERR_DTYPE;
  if (rows < 0 || rows > 2147483647LL || n_shard < 1 || n_shard > 2147483647LL || ldx < n_shard) return SPARK_ERR_SHAPE;
  if (y && ldy < n_shard) return SPARK_ERR_SHAPE;
  if (idx && idx_cap < 0) return SPARK_ERR_SHAPE;
  const size_t es = dtype_size(dt);
  if (!aligned16(x) || (ldx * es) % 16) return SPARK_ERR_ALIGN;
  if (y && (!aligned16(y) || (ldy * es) % 16)) return SPARK_ERR_ALIGN;
  const hipError_t e = spark::launch_stat_topk(x, dt == SPARK_BF16, rows, n_shard, ldx, 0.f, fill == SPARK_FILL_NEG_INF,
                                               0.f, y, ldy, nullptr, count, idx, idx_cap, nullptr,
                                               static_cast<hipStream_t>(hip_stream), theta, nullptr);
  return e == hipSuccess ? SPARK_OK : SPARK_ERR_DEVICE;
}

spark_status spark_stat_topk_huber(const void* x, spark_dtype dt, int64_t rows, int64_t n, int64_t ldx, int64_t k,
                                   float delta, void* y, int64_t ldy, float* theta, void* hip_stream) {
  if (!x || !y) return SPARK_ERR_NULL;
  if (!dtype_ok(dt)) return SPARK_ERR_DTYPE;
  if (rows < 0 || rows > 2147483647LL || n < 2 || n > 2147483647LL || ldx < n || ldy < n) return SPARK_ERR_SHAPE;
  if (!(delta >= 0.f) || std::isinf(delta)) return SPARK_ERR_SHAPE;
  if (k < 1 || k > n - 1) return SPARK_ERR_K;
  const size_t es = dtype_size(dt);
  if (!aligned16(x) || (ldx * es) % 16 || !aligned16(y) || (ldy * es) % 16) return SPARK_ERR_ALIGN;
  const float z = (float)spark_normal_quantile(1.0 - (double)k / (double)n);
  const hipError_t e = spark::launch_stat_topk(x, dt == SPARK_BF16, rows, n, ldx, z, 0, delta, y, ldy, theta, nullptr,
                                               nullptr, 0, nullptr, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? SPARK_OK : SPARK_ERR_DEVICE;
}

spark_status spark_stat_topk_huber_backward(const void* x, const void* gy, spark_dtype dt, int64_t rows, int64_t n,
                                            int64_t ldx, int64_t ldgy, int64_t k, float delta, void* gx,
                                            int64_t ldgx, void* hip_stream) {
  if (!x || !gy || !gx) return SPARK_ERR_NULL;
  if (!dtype_ok(dt)) return SPARK_ERR_DTYPE;
  if (rows < 0 || rows > 2147483647LL || n < 2 || n > 2147483647LL || ldx < n || ldgy < n || ldgx < n)
    return SPARK_ERR_SHAPE;
  if (!(delta >= 0.f) || std::isinf(delta)) return SPARK_ERR_SHAPE;
  if (k < 1 || k > n - 1) return SPARK_ERR_K;
  const size_t es = dtype_size(dt);
  if (!aligned16(x) || (ldx * es) % 16 || !aligned16(gy) || (ldgy * es) % 16 || !aligned16(gx) || (ldgx * es) % 16)
    return SPARK_ERR_ALIGN;
  const float z = (float)spark_normal_quantile(1.0 - (double)k / (double)n);
  const hipError_t e = spark::launch_stat_topk_vjp(x, gy, dt == SPARK_BF16, rows, n, ldx, ldgy, z, delta, gx, ldgx,
                                                   static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? SPARK_OK : SPARK_ERR_DEVICE;
}

size_t spark_ffn_workspace_bytes(int32_t d_model, int32_t d_ff, int32_t batch) {
  if (d_model < 2 || d_ff < 2 || batch < 1 || batch > SPARK_MAX_BATCH) return 0;
  return spark::ffn_workspace_bytes(d_model, d_ff, batch);
}

spark_status spark_ffn_decode(const spark_ffn_layer* layer, const void* q, spark_dtype qdtype, int32_t batch,
                              int64_t ldq, float* y, float* theta, int32_t* active_count,
                              int32_t* active_idx, int32_t* union_count, int32_t* union_idx,
                              void* workspace, size_t workspace_bytes, void* hip_stream) {
  return decode_layers(layer, layer ? 1 : 0, q, qdtype, batch, ldq, y, theta, active_count, active_idx, union_count,
                       union_idx, workspace, workspace_bytes, spark::FfnTuning(), static_cast<hipStream_t>(hip_stream));
}

spark_status spark_ffn_decode_static(const spark_ffn_layer* layer, const void* q, spark_dtype qdtype, int32_t batch,
                                     int64_t ldq, float* y, float* theta, int32_t* active_count,
                                     int32_t* active_idx, int32_t* union_count, int32_t* union_idx,
                                     void* hip_stream) {
  const spark_status s = validate_decode_args(layer, q, qdtype, batch, ldq, y);
  if (s != SPARK_OK) return s;
  if (batch != 1) return SPARK_ERR_SHAPE;
  const spark::FfnProblem p = make_problem(layer, q, qdtype, batch, ldq, y, theta, active_count, active_idx,
                                           union_count, union_idx);
  if (!spark::phased_supported(p)) return SPARK_ERR_SHAPE;
  if (spark::phased_scratch_bytes(layer->d_model, layer->d_ff, 1) > (size_t)SPARK_STATIC_SCRATCH_BYTES)
    return SPARK_ERR_WORKSPACE;
  const int part_rows = spark::phased_part_rows(SPARK_STATIC_SCRATCH_BYTES, layer->d_model, layer->d_ff, 1);
  void* ptr = nullptr;
  if (static_scratch_address(&ptr) != hipSuccess) return SPARK_ERR_DEVICE;
  // the same launches as spark_ffn_decode, on the built-in array laid out for one layer; every word
  // the kernels read from it they have written earlier in this call, so nothing needs clearing
  const hipError_t e = run_phased(layer, 1, p, spark::FfnTuning(), ptr, 1, part_rows, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? SPARK_OK : SPARK_ERR_DEVICE;
}

spark_status spark_ffn_decode_layers(const spark_ffn_layer* layers, int32_t n_layers, const void* q,
                                     spark_dtype qdtype, int32_t batch, int64_t ldq, float* y, float* theta,
                                     int32_t* active_count, int32_t* active_idx, int32_t* union_count,
                                     int32_t* union_idx, void* workspace, size_t workspace_bytes,
                                     void* hip_stream) {
  return decode_layers(layers, n_layers, q, qdtype, batch, ldq, y, theta, active_count, active_idx, union_count,
                       union_idx, workspace, workspace_bytes, spark::FfnTuning(), static_cast<hipStream_t>(hip_stream));
}

spark_status spark_ffn_decode_layers_tuned(const spark_ffn_layer* layers, int32_t n_layers, const void* q,
                                           spark_dtype qdtype, int32_t batch, int64_t ldq, float* y, float* theta,
                                           int32_t* active_count, int32_t* active_idx, int32_t* union_count,
                                           int32_t* union_idx, void* workspace, size_t workspace_bytes,
                                           const spark_ffn_tuning* tuning, void* hip_stream) {
  return decode_layers(layers, n_layers, q, qdtype, batch, ldq, y, theta, active_count, active_idx, union_count,
                       union_idx, workspace, workspace_bytes, make_tuning(tuning), static_cast<hipStream_t>(hip_stream));
}

size_t spark_ffn_prefill_workspace_bytes(int32_t d_model, int32_t d_ff, int32_t chunk) {
  size_t need = 0;  // a shorter last chunk may take another path with another scratch layout
  for (int32_t b = 1; b <= chunk; ++b) {
    const size_t w = spark_ffn_workspace_bytes(d_model, d_ff, b);
    if (w == 0) return 0;
    need = w > need ? w : need;
  }
  return need;
}

spark_status spark_ffn_prefill(const spark_ffn_layer* layer, const void* q, spark_dtype qdtype, int64_t n_tokens,
                               int32_t chunk, int64_t ldq, float* y, float* theta, int32_t* active_count,
                               int32_t* active_idx, int32_t* union_count, int32_t* union_idx, void* workspace,
                               size_t workspace_bytes, void* hip_stream) {
  if (n_tokens < 0 || n_tokens > 2147483647LL) return SPARK_ERR_SHAPE;
  const spark_status s = validate_decode(layer, q, qdtype, chunk, ldq, y, workspace, workspace_bytes);
  if (s != SPARK_OK) return s;
  if (workspace_bytes < spark_ffn_prefill_workspace_bytes(layer->d_model, layer->d_ff, chunk)) return SPARK_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const spark::FfnTuning tune;
  const int64_t d_model = layer->d_model, d_ff = layer->d_ff, n_full = n_tokens / chunk;
  const int32_t tail = (int32_t)(n_tokens % chunk);
  const size_t qs = dtype_size(qdtype);
  // outputs and tokens of the chunk that starts at token t0 (c = its chunk number)
  auto problem_at = [&](int64_t t0, int64_t c, int32_t batch) {
    return make_problem(layer, static_cast<const char*>(q) + (size_t)t0 * (size_t)ldq * qs, qdtype, batch, ldq,
                        y + t0 * d_model, theta ? theta + t0 : nullptr, active_count ? active_count + t0 : nullptr,
                        active_idx ? active_idx + t0 * d_ff : nullptr, union_count ? union_count + c : nullptr,
                        union_idx ? union_idx + c * d_ff : nullptr);
  };
  auto one_chunk = [&](int64_t t0, int64_t c, int32_t batch) {
    const spark::FfnProblem p = problem_at(t0, c, batch);
    const spark::FfnWorkspace ws = spark::carve_workspace(workspace, layer->d_model, layer->d_ff, batch);
    if (takes_phased(p, tune)) return run_phased(layer, 1, p, tune, ws.phased, spark::kPhasedMaxLayers, kWorkspacePartRows, st);
    return spark::launch_ffn_general(p, ws, 0, st);
  };
  int64_t c = 0;
  if (n_full > 0 && spark::phased_batch_supported(problem_at(0, 0, chunk))) {
    // the full chunks are independent of each other: they go through the batched path as the
    // "layers" of one launch, every slot with the same weights and its own block of tokens
    const spark::FfnWorkspace ws = spark::carve_workspace(workspace, layer->d_model, layer->d_ff, chunk);
    const void* w1[256];
    const void* w2[256];
    const void* w3[256];
    for (int i = 0; i < 256; ++i) {
      w1[i] = layer->k1n;
      w2[i] = layer->k2n;
      w3[i] = layer->vn;
    }
    for (; c < n_full; c += 256) {
      spark::FfnProblem p = problem_at(c * chunk, c, chunk);
      p.q_slot_stride = (int64_t)chunk * ldq;
      const int n = (int)(n_full - c < 256 ? n_full - c : 256);
      if (spark::launch_ffn_phased_batch(p, w1, w2, w3, n, tune, ws.phased, st) != hipSuccess) return SPARK_ERR_DEVICE;
    }
    c = n_full;
  }
  for (; c < n_full; ++c)
    if (one_chunk(c * chunk, c, chunk) != hipSuccess) return SPARK_ERR_DEVICE;
  if (tail > 0 && one_chunk(n_full * chunk, n_full, tail) != hipSuccess) return SPARK_ERR_DEVICE;
  return SPARK_OK;
}

spark_status spark_ffn_dense_decode(const spark_ffn_layer* layer, const void* q, spark_dtype qdtype,
                                    int32_t batch, int64_t ldq, float* y, void* workspace,
                                    size_t workspace_bytes, void* hip_stream) {
  const spark_status s = validate_decode(layer, q, qdtype, batch, ldq, y, workspace, workspace_bytes);
  if (s != SPARK_OK) return s;
  if (is_code_dtype(layer->wdtype)) return SPARK_ERR_DTYPE;  // use spark_ffn_dense_decode_layers
  const spark::FfnProblem p =
      make_problem(layer, q, qdtype, batch, ldq, y, nullptr, nullptr, nullptr, nullptr, nullptr);
  const spark::FfnWorkspace ws = spark::carve_workspace(workspace, layer->d_model, layer->d_ff, batch);
  const hipError_t e = spark::launch_ffn_general(p, ws, 1, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? SPARK_OK : SPARK_ERR_DEVICE;
}

spark_status spark_ffn_dense_decode_layers(const spark_ffn_layer* layers, int32_t n_layers, const void* q,
                                           spark_dtype qdtype, int32_t batch, int64_t ldq, float* y,
                                           void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!layers) return SPARK_ERR_NULL;
  if (n_layers < 1) return SPARK_ERR_SHAPE;
  for (int32_t l = 0; l < n_layers; ++l) {
    const spark_status s = validate_decode(&layers[l], q, qdtype, batch, ldq, y, workspace, workspace_bytes);
    if (s != SPARK_OK) return s;
    if (layers[l].d_model != layers[0].d_model || layers[l].d_ff != layers[0].d_ff ||
        layers[l].r != layers[0].r || layers[l].k != layers[0].k || layers[l].wdtype != layers[0].wdtype ||
        layers[l].gelu != layers[0].gelu)
      return SPARK_ERR_SHAPE;
  }
  if (is_code_dtype(layers[0].wdtype) && batch != 1) return SPARK_ERR_DTYPE;  // dense comparison of 8-bit weights: one token
  const int64_t d_model = layers[0].d_model;
  const spark::FfnWorkspace ws = spark::carve_workspace(workspace, layers[0].d_model, layers[0].d_ff, batch);
  const spark::FfnProblem p0 =
      make_problem(&layers[0], q, qdtype, batch, ldq, y, nullptr, nullptr, nullptr, nullptr, nullptr);
  if (spark::phased_supported(p0)) {
    const hipError_t e = run_phased(layers, n_layers, p0, spark::FfnTuning(), ws.phased, spark::kPhasedMaxLayers,
                                    kWorkspacePartRows, static_cast<hipStream_t>(hip_stream), 1);
    return e == hipSuccess ? SPARK_OK : SPARK_ERR_DEVICE;
  }
  for (int32_t l = 0; l < n_layers; ++l) {
    const spark::FfnProblem p = make_problem(&layers[l], q, qdtype, batch, ldq, y + (int64_t)l * batch * d_model,
                                             nullptr, nullptr, nullptr, nullptr, nullptr);
    if (spark::launch_ffn_general(p, ws, 1, static_cast<hipStream_t>(hip_stream)) != hipSuccess) return SPARK_ERR_DEVICE;
  }
  return SPARK_OK;
}

size_t spark_attn_workspace_bytes(int32_t n_heads, int32_t group, int32_t n_ctx) {
  if (n_heads < 1 || group < 1 || group > 4 || n_ctx < 1 || n_ctx > spark::kAttnMaxCtx) return 0;
  return spark::attn_workspace_bytes(n_heads, group, n_ctx);
}

spark_status spark_attn_decode(const spark_attn_head* heads, int32_t n_heads, const void* q, spark_dtype qdtype,
                               float* y, float* theta, int32_t* kept_count, int32_t* kept_idx, void* workspace,
                               size_t workspace_bytes, void* hip_stream) {
  if (!heads || !q || !y) return SPARK_ERR_NULL;
  if (n_heads < 1) return SPARK_ERR_SHAPE;
  if (!dtype_ok(qdtype)) return SPARK_ERR_DTYPE;
  const spark_attn_head& h0 = heads[0];
  for (int32_t i = 0; i < n_heads; ++i) {
    const spark_attn_head& h = heads[i];
    if (!h.k1c || !h.k2c || !h.vc) return SPARK_ERR_NULL;
    if (!dtype_ok(h.cdtype)) return SPARK_ERR_DTYPE;
    if (h.n_ctx != h0.n_ctx || h.d_attn != h0.d_attn || h.r != h0.r || h.k != h0.k || h.cdtype != h0.cdtype ||
        h.group != h0.group)
      return SPARK_ERR_SHAPE;
    if (!aligned16(h.k1c) || !aligned16(h.k2c) || !aligned16(h.vc)) return SPARK_ERR_ALIGN;
  }
  if (h0.n_ctx < 1 || h0.d_attn < 2 || h0.r < 1 || h0.r > h0.d_attn - 1) return SPARK_ERR_SHAPE;
  if (h0.k < 1) return SPARK_ERR_K;
  spark::AttnProblem p;
  p.n_ctx = h0.n_ctx;
  p.d_attn = h0.d_attn;
  p.r = h0.r;
  p.k = h0.k;
  p.group = h0.group;
  p.c_bf16 = h0.cdtype == SPARK_BF16;
  p.q_bf16 = qdtype == SPARK_BF16;
  p.z = h0.n_ctx > h0.k ? (float)spark_normal_quantile(1.0 - (double)h0.k / (double)h0.n_ctx) : 0.f;
  p.q = q;
  p.y = y;
  p.theta = theta;
  p.count = kept_count;
  p.idx = kept_idx;
  if (!spark::attn_supported(p)) return SPARK_ERR_SHAPE;
  if (!aligned16(q) || (h0.r * dtype_size(qdtype)) % 16 || (h0.d_attn * dtype_size(qdtype)) % 16) return SPARK_ERR_ALIGN;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return SPARK_ERR_WORKSPACE;
  if (workspace_bytes < spark_attn_workspace_bytes(n_heads, h0.group, h0.n_ctx)) return SPARK_ERR_WORKSPACE;
  const void* k1c[spark::kAttnMaxHeads];
  const void* k2c[spark::kAttnMaxHeads];
  const void* vc[spark::kAttnMaxHeads];
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  for (int32_t base = 0; base < n_heads; base += spark::kAttnMaxHeads) {
    const int32_t n = n_heads - base < spark::kAttnMaxHeads ? n_heads - base : spark::kAttnMaxHeads;
    for (int32_t i = 0; i < n; ++i) {
      k1c[i] = heads[base + i].k1c;
      k2c[i] = heads[base + i].k2c;
      vc[i] = heads[base + i].vc;
    }
    spark::AttnProblem pc = p;
    const size_t hg0 = (size_t)base * p.group;
    pc.q = static_cast<const char*>(q) + hg0 * p.d_attn * dtype_size(qdtype);
    pc.y = y + hg0 * p.d_attn;
    pc.theta = theta ? theta + hg0 : nullptr;
    pc.count = kept_count ? kept_count + hg0 : nullptr;
    pc.idx = kept_idx ? kept_idx + hg0 * p.n_ctx : nullptr;
    if (spark::launch_attn_decode(pc, k1c, k2c, vc, n, workspace, st) != hipSuccess) return SPARK_ERR_DEVICE;
  }
  return SPARK_OK;
}

size_t spark_stat_topk_workspace_bytes(int64_t rows, int64_t n) {
  (void)rows;
  (void)n;
  return 0;  // the row-wise kernels keep a row on chip: no scratch memory
}

spark_status spark_copy_bytes(void* dst, const void* src, size_t nbytes, void* hip_stream) {
  if (nbytes == 0) return SPARK_OK;
  if (!dst || !src) return SPARK_ERR_NULL;
  if (!aligned16(dst) || !aligned16(src) || nbytes % 16) return SPARK_ERR_ALIGN;
  const hipError_t e = spark::launch_copy_bytes(dst, src, nbytes, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? SPARK_OK : SPARK_ERR_DEVICE;
}

}  // extern "C"
