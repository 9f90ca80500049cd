// Host-side launchers of the Spark-FFN kernels (internal to the library).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace spark {

// Row-wise statistical top-k.  dt: 0 = fp32, 1 = bf16.  `flags`, when given, receives a 1 at
// every active column (used to form the union of the active sets of a batch).
// delta > 0: the kept entries are mapped through Huber(.; delta) / delta (0: plain soft threshold)
hipError_t launch_stat_topk(const void* x, int dt, int64_t rows, int64_t n, int64_t ldx, float z,
                            int fill, float delta, void* y, int64_t ldy, float* theta, int32_t* count,
                            int32_t* idx, int64_t idx_cap, int32_t* flags, hipStream_t st,
                            const float* theta_in = nullptr, float* stats_out = nullptr);
// (theta_in: per-row thresholds to apply instead of computing them; stats_out: [rows][2] (mean, centred
// sum of squares), after which the launch stops)
// thresholds from the shards' statistics stats[m][rows][2] with ns[m] entries per shard (host array)
hipError_t launch_combine_shard_stats(const float* stats, const int64_t* ns, int m, int64_t rows, float z, float* theta,
                                      float* mean_out, float* std_out, hipStream_t st);
// gx = gy . d(Huber(StatTop_k(x); delta) / delta)/dx, row by row
hipError_t launch_stat_topk_vjp(const void* x, const void* gy, int dt, int64_t rows, int64_t n, int64_t ldx,
                                int64_t ldgy, float z, float delta, void* gx, int64_t ldgx, hipStream_t st);

struct FfnProblem {
  int d_model, d_ff, r, k;
  int w_bf16, q_bf16, gelu;
  int w_fp8 = 0;  // 1: weights are OCP E4M3 codes, 2: signed 8-bit integers; every array followed by one fp32
                  // scale per row (batch-1 phased path only)
  const void *k1n, *k2n, *vn;
  const void* q;
  int64_t ldq;
  int64_t q_slot_stride = 0;  // batched multi-layer launches: elements between the token blocks of
                              // consecutive layer slots (0: every slot reads the same tokens)
  int batch;
  float z;  // Q(1 - k/d_ff)
  // outputs (optional ones may be null)
  float* y;
  float* theta;
  int32_t* active_count;
  int32_t* active_idx;
  int32_t* union_count;
  int32_t* union_idx;
};

// Carving of the caller's workspace.
struct FfnWorkspace {
  float* S;          // [batch][d_ff] predictor scores
  float* A;          // [batch][d_ff] StatTop_k(S)
  int32_t* flags;    // [d_ff] union membership
  int32_t* uidx;     // [d_ff] ascending union
  int32_t* ucount;   // [16]
  float* uact;       // [d_ff][batch] GELU(a) * g per union row
  float* part;       // [ksplit][batch][d_model] split partial sums of y
  int ksplit;
  void* phased;      // scratch of the phase-by-phase paths
  size_t phased_bytes;
};

size_t ffn_workspace_bytes(int d_model, int d_ff, int batch);
FfnWorkspace carve_workspace(void* base, int d_model, int d_ff, int batch);

// General path: separate kernels, any batch <= 64.  dense != 0 reads every K2 / V row.
hipError_t launch_ffn_general(const FfnProblem& p, const FfnWorkspace& ws, int dense, hipStream_t st);

// Per-call choices a caller may pin instead of leaving them to the library (all 0 = automatic);
// mirrors spark_ffn_tuning of the C ABI.
struct FfnTuning {
  int path = 0;     // 1: the general multi-kernel path even where a phase-by-phase path exists
  int phases = 0;   // batch-1 path: bit 0 predictor sweep, bit 1 gather, bit 2 reduction / index lists; 0 = all
  int rows_per_predict_block = 0;
  int neurons_per_gather_block = 0;
  int variant = 0;  // batch 1: 1 = the 8-wave gather; batches: row slices of the V step, +100 k-split kernels
                    // for every batch size, +200 streamed kernels however small the launch
};

// Phase-by-phase batch-1 path: predictor sweep, gather, reduce as ordinary launches over up
// to `layer_cap` (<= kPhasedMaxLayers) layers at a time (longer stacks are chained).  `scratch`
// is 256-byte aligned, needs no initialisation and has room for `part_rows` partial output rows
// (>= layer_cap) behind the scores and block statistics: phased_scratch_bytes gives the size with 64
// partial rows per layer of the cap, phased_part_rows the rows (at most 128 per layer) that a scratch
// of a given size holds.
constexpr int kPhasedMaxLayers = 64;
size_t phased_scratch_bytes(int d_model, int d_ff, int layer_cap);
int phased_part_rows(size_t scratch_bytes, int d_model, int d_ff, int layer_cap);
bool phased_supported(const FfnProblem& p);
hipError_t launch_ffn_phased(const FfnProblem& p0, const void* const* k1n, const void* const* k2n,
                             const void* const* vn, int n_layers, int dense, const FfnTuning& tune, void* scratch,
                             int layer_cap, int part_rows, hipStream_t st);

// Phase-by-phase path for batches of 2..64 tokens on the matrix cores (bf16 weights and
// tokens), up to kBatchMaxLayers layers per set of launches.
constexpr int kBatchMaxLayers = 32;
size_t phased_batch_scratch_bytes(int d_model, int d_ff, int batch);
bool phased_batch_supported(const FfnProblem& p);
hipError_t launch_ffn_phased_batch(const FfnProblem& p0, const void* const* k1n, const void* const* k2n,
                                   const void* const* vn, int n_layers, const FfnTuning& tune, void* scratch,
                                   hipStream_t st);

// A plain device-to-device copy kernel of known size (the reference the HBM byte counters are
// scaled by when traffic is measured).
hipError_t launch_copy_bytes(void* dst, const void* src, size_t nbytes, hipStream_t st);

// Spark-attention decode: one query per head over token-major caches, all heads of a call
// in two launches (up to kAttnMaxHeads caches per pair of launches; longer lists are chained).
constexpr int kAttnMaxHeads = 128;
constexpr int kAttnMaxCtx = 16384;
struct AttnProblem {
  int n_ctx, d_attn, r, k, group;
  int c_bf16, q_bf16;
  float z;          // Q(1 - k / n_ctx) (unused when n_ctx <= k)
  const void* q;    // [n_heads][group][d_attn]
  float* y;         // [n_heads][group][d_attn]
  float* theta;     // [n_heads][group]         optional
  int32_t* count;   // [n_heads][group]         optional
  int32_t* idx;     // [n_heads][group][n_ctx]  optional
};
bool attn_supported(const AttnProblem& p);
size_t attn_workspace_bytes(int n_heads, int group, int n_ctx);
hipError_t launch_attn_decode(const AttnProblem& p, const void* const* k1c, const void* const* k2c,
                              const void* const* vc, int n_heads, void* workspace, hipStream_t st);

}  // namespace spark
