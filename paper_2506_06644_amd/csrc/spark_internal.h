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
                            int32_t* idx, int64_t idx_cap, int32_t* flags, hipStream_t st);
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
  void* fused;       // scratch of the persistent batch-1 kernel
  size_t fused_bytes;
};

size_t ffn_workspace_bytes(int d_model, int d_ff, int batch);
FfnWorkspace carve_workspace(void* base, int d_model, int d_ff, int batch);

// General path: separate kernels, any batch <= 64.  dense != 0 reads every K2 / V row.
hipError_t launch_ffn_general(const FfnProblem& p, const FfnWorkspace& ws, int dense, hipStream_t st);

// Persistent batch-1 path: one launch for up to kFusedMaxLayers layers (longer stacks are
// chained).  `scratch` is ws.fused (fused_scratch_bytes(d_model, d_ff) bytes, 256-byte aligned); its
// first int32 is a status word the launch clears and sets non-zero if it had to abort.
constexpr int kFusedMaxLayers = 64;
size_t fused_scratch_bytes(int d_model, int d_ff);
void fused_set_profile(int on);               // testing aid: per-wave wait-time counters
size_t fused_profile_offset(int d_model, int d_ff);     // byte offset of the counters inside the scratch
size_t fused_profile_bytes();
bool fused_supported(const FfnProblem& p, int n_layers);
hipError_t launch_ffn_fused(const FfnProblem& p0, const void* const* k1n, const void* const* k2n,
                            const void* const* vn, int n_layers, void* scratch, hipStream_t st);

// Phase-by-phase batch-1 path: predictor sweep, gather, reduce as ordinary launches over up
// to kPhasedMaxLayers layers at a time (longer stacks are chained).  `scratch` holds
// phased_scratch_bytes(d_model, d_ff) bytes, 256-byte aligned, and needs no initialisation.
constexpr int kPhasedMaxLayers = 64;
size_t phased_scratch_bytes(int d_model, int d_ff);
bool phased_supported(const FfnProblem& p);
void phased_set_phases(int mask);  // measurement aid: bit 0 predict, bit 1 gather, bit 2 reduce / select; 0 = all
void phased_set_tuning(int rows_per_predict_block, int neurons_per_gather_block, int alt);  // 0 = automatic
hipError_t launch_ffn_phased(const FfnProblem& p0, const void* const* k1n, const void* const* k2n,
                             const void* const* vn, int n_layers, int dense, void* scratch, hipStream_t st);

// Phase-by-phase path for batches of 2..64 tokens on the matrix cores (bf16 weights and
// tokens), up to kBatchMaxLayers layers per set of launches.
constexpr int kBatchMaxLayers = 32;
size_t phased_batch_scratch_bytes(int d_model, int d_ff, int batch);
bool phased_batch_supported(const FfnProblem& p);
void phased_batch_set_tuning(int predict_tiles_per_workgroup, int k2_tiles_per_workgroup, int v_row_slices);  // 0 = automatic
hipError_t launch_ffn_phased_batch(const FfnProblem& p0, const void* const* k1n, const void* const* k2n,
                                   const void* const* vn, int n_layers, void* scratch, hipStream_t st);

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
