// Spark-FFN decode (Eq.2 of arXiv 2506.06644) for a batch of 2..64 tokens and a stack of
// independent layers, phase by phase over the whole stack, on the matrix cores of gfx950
// (bf16 or 8-bit weights and bf16 tokens; Appendix B's batching: every token has its own threshold and
// mask, the union of the masks decides which weight rows are fetched).
//
//   predict   S[l][b][j] = K1n_l[j] . q_b[:r].  Three kernel families, chosen per call: with at
//             most 16 tokens a wave reads four rows whole and multiplies on the 4x4x4 matrix
//             instruction (tokens in LDS); with more, 16-row tiles are staged in LDS by whole-row
//             loads and multiplied with v_mfma_f32_16x16x32_bf16 by waves that hold the tokens
//             of one token block and one part of the k range in registers; every other shape
//             takes the first version's kernels, which split the k range over 8 or 10 loader
//             waves that read MFMA-shaped pieces.
//   select    one workgroup per (layer, token): mean and std of the row (two passes over
//             registers), theta (Eq.11), the token's index list and the token's mask; a small
//             launch then ORs the tokens' masks of a layer and lists the union's neurons.
//   k2        G[m][b] = K2n[U[m]] . q_b[r:] over the union's rows (the same three families),
//             u[m][b] = GELU(s_bj - theta_b) * G (0 where token b does not activate the row),
//             stored token-major as bf16 planes: three (u = p0 + p1 + p2 carries all 24
//             significant bits of the fp32 value) up to 16 tokens, two above.
//   v         y[b][c] += sum_m u[m][b] * Vn[U[m]][c]: the contraction runs over rows while Vn
//             is contiguous along columns, so each wave stages its 32 rows x 64 columns
//             through LDS and reads them back transposed (8 consecutive rows of one column
//             per lane), then v_mfma_f32_16x16x32_bf16 with tokens as M and columns as N.
//             Row slices give partial outputs.
//   reduce    y = sum of the partial outputs in slice order.
//
// 8-bit weight codes (E4M3 or integers with a scale per row) are widened to bf16, which holds
// them exactly, in registers or on the way into LDS, by the first two families and the v step.
//
// bf16 x bf16 products are exact in fp32 and all accumulation is fp32.  Nothing waits on
// another workgroup inside a launch, and every sum has a fixed order.
#include "spark_device.h"
#include "spark_internal.h"

namespace spark {

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

constexpr int kRowWavesAll = 12;  // waves of a predict / k2 workgroup: NLW loaders (k split) + the rest emit
constexpr int kVPitch = 160;     // bytes between row positions of a staged V tile (conflict-free transposed reads)
constexpr int kMaxPlanes = 3;    // bf16 planes of u: 3 x 8 significant bits carry an fp32 value
// Planes a call uses: all three with one token block; two (16 significant bits, a relative
// error of 2^-17 per activation, far inside the bf16-weight tolerance) with more, where the
// V step's matrix work per byte is highest and the third plane costs a tenth of the call.
constexpr int planes_for(int nb) { return nb == 1 ? 3 : 2; }
constexpr int kMaxWords = 256;   // 64-bit union mask words per layer: d_ff <= 16384

struct BatchParams {
  const void* k1n[kBatchMaxLayers];
  const void* k2n[kBatchMaxLayers];
  const void* vn[kBatchMaxLayers];
  const bf16_t* q;     // [B][ldq]; layer slot l reads the block at q + l * qslot
  int64_t ldq;
  int64_t qslot;
  float* y;            // [L][B][d_model]
  float* theta;        // [L][B]        optional
  int32_t* count;      // [L][B]        optional
  int32_t* idx;        // [L][B][d_ff]  optional
  int32_t* ucount;     // [L]           optional
  int32_t* uidx;       // [L][d_ff]     optional
  float* S;                    // [L][B][d_ff]  predictor scores, token-major (read by select)
  float* ST;                   // [L][d_ff][BP] the same, neuron-major (read by k2: one 64-byte piece per row and token block)
  float* thetas;               // [L][B]
  unsigned long long* tmask;   // [L][B][kMaxWords]  mask of every token
  int32_t* urow;               // [L][d_ff]       union rank -> neuron
  int32_t* utotal;             // [L]             union size
  uint16_t* up;                // [planes][L][ldu / 8][B][8]  bf16 planes of u (u = sum of the planes): union ranks in
                               // blocks of 8, so that the 8 consecutive ranks of one token the v phase feeds to a lane
                               // are 16 contiguous bytes and a group's tokens are contiguous too
  size_t plane;                // elements between planes
  float* part;                 // [L][KS][B][d_model]
  int n_layers, B, BP, d_model, d_ff, r, gelu, ldu;  // BP = B rounded up to 16
  int planes;  // bf16 planes of u in use
  float z;
  int TPW1;  // predict tiles per workgroup (even)
  int TPW2;  // k2 tiles per workgroup (even, <= 32)
  int KS;    // row slices of the v phase
  int VSLABS;  // column slabs of the v phase
};

__device__ __forceinline__ u32x4 ld16(const void* p) { return *reinterpret_cast<const u32x4*>(p); }
__device__ __forceinline__ u32x4 ld16_stream(const void* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
}
__device__ __forceinline__ f32x4 mfma_bf16(u32x4 a, u32x4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}
// Workgroup barrier that orders LDS traffic only.  __syncthreads() also fences global memory,
// i.e. waits for every outstanding global load of the wave, which would drain the very
// prefetch that is meant to stay in flight across the barrier.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}
// k step (of 32) that wave `w` takes as its s-th: steps are dealt in pairs so that a wave
// reads whole 128-byte lines of a row
template <int SPW, int NLW> __device__ __forceinline__ int k_step_t(int s, int w) { return (s >> 1) * 2 * NLW + 2 * w + (s & 1); }

// ---------------------------------------------------------------------------- rows x tokens
// Shared by predict (rows are the neurons 16 * tile + i) and k2 (rows are union ranks, looked up
// in `rowidx`).  A workgroup has NLW LOADER waves (8 or 10, whichever
// covers the k steps with fewer registers) and 12 - NLW EMIT waves.
//
// Loader wave w owns the k steps k_step(s, w): it holds the token fragments of those steps in
// registers, keeps DEPTH tiles of its row slices in flight, multiplies, and leaves its partial
// tile in LDS.  Its loop contains no store and no branch: on this target stores share the
// loads' counter and a wave with both kinds pending can only wait for all of them, so a
// store in this loop would drain the prefetch at every tile.  A tile past `tile_end` is
// requested through a buffer descriptor without records: the loads are issued all the same
// (their number in flight stays a compile-time constant, the waits are exact) but touch no
// memory.
//
// Emit wave e sums the loaders' partials of the token blocks e, e + kEmitWaves, ... in loader
// order and hands the four values D[row 4 * kg + i][token nb * 16 + ri], i < 4, that a lane
// holds of a block to `emit(tile, nb, values, side)`, which stores them (four consecutive rows
// of one token per lane: 16- or 8-byte stores).  With HAS_SIDE, `side` holds a value per (row,
// lane) that the emit wave fetched two tiles ahead with `pre(tile, nb, i)` (fetched by the loaders instead, these
// small scattered loads sit in front of the weight rows in the in-order return queue and cost
// a third of the kernel).  One LDS-only barrier per tile; the partial buffers alternate,
// and a loader that writes a buffer again two tiles later has passed the barrier of the tile
// in between, which the emit waves reach only after they have finished reading it.
constexpr int kRowThreads = kRowWavesAll * kWave;
template <int NB, int SPW>
constexpr int tile_depth() { return 2; }  // tiles in flight per loader wave (deeper did not pay: see the notes on measurements)  // DEPTH * SPW * 4 registers hold the tiles in flight
template <int NB>
constexpr size_t rows_lds_bytes() { return (size_t)2 * 10 * NB * 4 * kWave * sizeof(float); }
template <int NB, int SPW, int NLW, bool HAS_SIDE, typename RowOf, typename Pre, typename Emit>
__device__ __forceinline__ void rows_times_tokens(const bf16_t* __restrict__ w, uint32_t w_bytes, int K,
                                                  const bf16_t* __restrict__ q, int64_t ldq, int qoff, int B,
                                                  int tile0, int ntiles, int tile_end,
                                                  float* red_raw, RowOf row_of, Pre pre, Emit emit) {
  constexpr int kRowWaves = NLW, kEmitWaves = kRowWavesAll - NLW;
  constexpr int NBE = (NB + kEmitWaves - 1) / kEmitWaves;  // token blocks an emit wave handles per tile
  float(*red)[kRowWaves][NB * 4][kWave] = reinterpret_cast<float(*)[kRowWaves][NB * 4][kWave]>(red_raw);
  constexpr int DEPTH = tile_depth<NB, SPW>();
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int kg = lane >> 4, ri = lane & 15;
  if (wave >= kRowWaves) {
    // ------------------------------------------------------------------ emit wave
    const int ew = wave - kRowWaves;
    float side[2][NBE][4];
    auto prefetch = [&](int t, float(&sv)[NBE][4]) {
      if constexpr (HAS_SIDE) {
#pragma unroll
        for (int k = 0; k < NBE; ++k)
#pragma unroll
          for (int e = 0; e < 4; ++e) sv[k][e] = pre(t, min(ew + kEmitWaves * k, NB - 1), e);
      }
    };
    auto emit_tile = [&](int i, const float(&sv)[NBE][4]) {
      const int buf = i & 1;
      lds_barrier();
#pragma unroll
      for (int k = 0; k < NBE; ++k) {
        const int nb = ew + kEmitWaves * k;
        if (nb < NB) {
          f32x4 v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int wv = 0; wv < kRowWaves; ++wv) v[e] += red[buf][wv][nb * 4 + e][lane];
          emit(tile0 + i, nb, v, f32x4{sv[k][0], sv[k][1], sv[k][2], sv[k][3]});
        }
      }
    };
    prefetch(tile0, side[0]);
    prefetch(tile0 + 1, side[1]);
    for (int i = 0; i < ntiles; i += 2) {  // ntiles is even
      emit_tile(i, side[0]);
      prefetch(tile0 + i + 2, side[0]);
      emit_tile(i + 1, side[1]);
      prefetch(tile0 + i + 3, side[1]);
    }
    return;
  }
  // -------------------------------------------------------------------- loader wave
  const int nsteps = K / 32;
  u32x4 qf[SPW][NB];
#pragma unroll
  for (int s = 0; s < SPW; ++s) {
    const int ks = k_step_t<SPW, NLW>(s, wave);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const int b = nb * 16 + ri;
      const bool ok = ks < nsteps && b < B;
      qf[s][nb] = ld16(q + (int64_t)(b < B ? b : 0) * ldq + qoff + ((ks < nsteps ? ks : 0) * 4 + kg) * 8);
      if (!ok) qf[s][nb] = u32x4{0u, 0u, 0u, 0u};
    }
  }
  auto load_tile = [&](int t, u32x4(&a)[SPW]) {
    const __amdgpu_buffer_rsrc_t rs =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(w), 0, t < tile_end ? (int)w_bytes : 0, 0x00020000);
    const uint32_t row_off = (uint32_t)row_of(t, ri) * (uint32_t)K * 2u;
#pragma unroll
    for (int s = 0; s < SPW; ++s) {
      const int ks = k_step_t<SPW, NLW>(s, wave);  // steps past K meet a zero token fragment
      a[s] = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)(row_off + (uint32_t)((ks < nsteps ? ks : 0) * 4 + kg) * 16u), 0, 0);
    }
  };
  auto process = [&](const u32x4(&a)[SPW], int buf) {
    f32x4 acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < SPW; ++s)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) acc[nb] = mfma_bf16(a[s], qf[s][nb], acc[nb]);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int e = 0; e < 4; ++e) red[buf][wave][nb * 4 + e][lane] = acc[nb][e];
    lds_barrier();
  };
  u32x4 a[DEPTH][SPW];
#pragma unroll
  for (int d = 0; d < DEPTH; ++d) load_tile(tile0 + d, a[d]);
  for (int i = 0; i < ntiles; i += DEPTH) {  // ntiles is a multiple of DEPTH (an even number)
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
      process(a[d], d & 1);
      load_tile(tile0 + i + d + DEPTH, a[d]);
    }
  }
}

// 8-bit weight codes (WK = 1: OCP E4M3, 2: signed integers): the 16 codes of one 16-byte piece
// widened to bf16, which holds both kinds exactly (an E4M3 value has 4 significant bits, an
// integer up to 127 has 7), as 8 words in element order.  The row's scale is applied to the
// finished dot product by the caller.
template <int WK>
__device__ __forceinline__ void codes_to_bf16(u32x4 a, uint32_t (&o)[8]) {
  typedef float f32x2_v __attribute__((ext_vector_type(2)));
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    float f[4];
    if constexpr (WK == 1) {
      const f32x2_v lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)a[d], false), hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)a[d], true);
      f[0] = lo[0]; f[1] = lo[1]; f[2] = hi[0]; f[3] = hi[1];
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) f[e] = (float)(int)(int8_t)(a[d] >> (8 * e));
    }
    // (the upper halves of two floats side by side: truncation is exact here)
    o[2 * d] = __builtin_amdgcn_perm(__float_as_uint(f[1]), __float_as_uint(f[0]), 0x07060302u);
    o[2 * d + 1] = __builtin_amdgcn_perm(__float_as_uint(f[3]), __float_as_uint(f[2]), 0x07060302u);
  }
}

// ------------------------------------------------- rows x tokens, tiles staged in LDS (> 16 tokens)
// The k-split kernels above read a tile of 16 rows in 64- and 128-byte pieces, one piece per
// row and instruction, which the memory system serves well below what whole rows reach.  Here
// the COMPUTE waves (2, 4 or 8 per token block: wave (nb, h) multiplies part h of every row by the
// tokens of block nb, whose operands it keeps in registers) first bring each tile into LDS with
// whole-row nontemporal loads: a wave fetches 16 / NCW consecutive rows, 256 or 512 contiguous
// bytes of each per instruction, two tiles ahead, and parks a tile in LDS one step before it is
// multiplied.  Every compute wave then reads its part of all 16 rows from LDS as the A operand.
// The parts' sums meet in LDS, where the EMIT waves (2 or 4) add them and
// store, exactly as above.  One LDS-only barrier per tile.  LDS: two tiles of 16 x (2 K + 16)
// bytes (the 16 bytes spread the rows over the banks) and two buffers of partial sums.
template <int CJ>
constexpr int staged_pitch() { return CJ * 512 + 16; }  // bytes between rows of a tile in LDS (K = 256 CJ)
// k parts a row is split into among the compute waves of a token block, and the waves of a
// workgroup: KP NB compute waves (4 or 8: they stage 16 / (KP NB) rows each) plus the emit waves.
constexpr int staged_parts(int nb, int cj) { return nb == 1 ? (cj <= 5 ? 4 : 8) : nb == 2 ? (cj <= 4 ? 2 : 4) : 2; }
constexpr int staged_emit_waves(int nb) { return nb >= 4 ? 4 : 2; }
constexpr int staged_waves(int nb, int cj) { return staged_parts(nb, cj) * nb + staged_emit_waves(nb); }
template <int NB, int CJ>
constexpr size_t staged_lds_bytes() {
  return (size_t)2 * 16 * staged_pitch<CJ>() + (size_t)2 * staged_parts(NB, CJ) * NB * 4 * kWave * sizeof(float) + 4 * 16 * sizeof(float);
}
// WK != 0: the rows are 8-bit codes (K bytes each); they are widened to bf16 when a tile is parked,
// so the tile in LDS and the multiplies are the same, and scale_of(row) (the row's scale, fetched
// with the row by the lane that stages its first piece) reaches the emit waves through LDS.
template <int WK, int NB, int CJ, bool HAS_SIDE, typename RowOf, typename ScaleOf, typename Pre, typename Emit>
__device__ __forceinline__ void rows_times_tokens_staged(const void* __restrict__ w, uint32_t w_bytes,
                                                         const bf16_t* __restrict__ q, int64_t ldq, int qoff, int B,
                                                         int tile0, int ntiles, int tile_end, unsigned char* lds,
                                                         RowOf row_of, ScaleOf scale_of, Pre pre, Emit emit) {
  constexpr int K = 256 * CJ, PITCH = staged_pitch<CJ>(), TILE = 16 * PITCH;
  constexpr int KP = staged_parts(NB, CJ);
  constexpr int NCW = KP * NB, kEmitWaves = staged_emit_waves(NB);
  constexpr int NBE = (NB + kEmitWaves - 1) / kEmitWaves;
  constexpr int HS = 8 * CJ / KP;       // k steps (of 32) per part of a row
  constexpr int RPWV = 16 / NCW;        // rows a compute wave stages per tile
  constexpr int LPR = kWave / RPWV;     // lanes per staged row
  constexpr int ROWB = WK ? K : 2 * K;  // bytes of a row in memory
  constexpr int NPC = ROWB / 16;        // its 16-byte pieces
  constexpr int NLD = (NPC + LPR - 1) / LPR;  // 16-byte loads per lane and tile
  static_assert(NCW == 4 || NCW == 8, "the compute waves share the 16 rows of a tile evenly");
  float(*red)[KP][NB * 4][kWave] = reinterpret_cast<float(*)[KP][NB * 4][kWave]>(lds + 2 * TILE);
  float(*sc_sh)[16] = reinterpret_cast<float(*)[16]>(lds + 2 * TILE + sizeof(float) * 2 * KP * NB * 4 * kWave);
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int kg = lane >> 4, ri = lane & 15;
  if (wave >= NCW) {
    // ------------------------------------------------------------------ emit wave
    const int ew = wave - NCW;
    float side[2][NBE][4];
    auto prefetch = [&](int t, float(&sv)[NBE][4]) {
      if constexpr (HAS_SIDE) {
#pragma unroll
        for (int k = 0; k < NBE; ++k)
#pragma unroll
          for (int e = 0; e < 4; ++e) sv[k][e] = pre(t, min(ew + kEmitWaves * k, NB - 1), e);
      }
    };
    auto emit_tile = [&](int i, const float(&sv)[NBE][4]) {
      const int buf = i & 1;
      lds_barrier();
#pragma unroll
      for (int k = 0; k < NBE; ++k) {
        const int nb = ew + kEmitWaves * k;
        if (nb < NB) {
          f32x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            v[e] = red[buf][0][nb * 4 + e][lane];
#pragma unroll
            for (int part = 1; part < KP; ++part) v[e] += red[buf][part][nb * 4 + e][lane];
            if constexpr (WK != 0) v[e] *= sc_sh[i & 3][4 * kg + e];
          }
          emit(tile0 + i, nb, v, f32x4{sv[k][0], sv[k][1], sv[k][2], sv[k][3]});
        }
      }
    };
    prefetch(tile0, side[0]);
    prefetch(tile0 + 1, side[1]);
    lds_barrier();  // (the compute waves' opening barrier: the first tile is in LDS)
    for (int i = 0; i < ntiles; i += 2) {  // ntiles is even
      emit_tile(i, side[0]);
      prefetch(tile0 + i + 2, side[0]);
      emit_tile(i + 1, side[1]);
      prefetch(tile0 + i + 3, side[1]);
    }
    return;
  }
  // ------------------------------------------------------------------- compute wave
  const int nbw = wave / KP, h = wave % KP;
  u32x4 qf[HS];
#pragma unroll
  for (int s = 0; s < HS; ++s) {
    const int b = nbw * 16 + ri;
    qf[s] = ld16(q + (int64_t)(b < B ? b : 0) * ldq + qoff + ((h * HS + s) * 4 + kg) * 8);
    if (b >= B) qf[s] = u32x4{0u, 0u, 0u, 0u};
  }
  const int srow = wave * RPWV + lane % RPWV, piece = lane / RPWV;  // the row of the tile this lane stages
  auto load_stage = [&](int t, u32x4(&st)[NLD], float& sc) {  // tiles past tile_end: a descriptor without records
    const __amdgpu_buffer_rsrc_t rs =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(w), 0, t < tile_end ? (int)w_bytes : 0, 0x00020000);
    const int row = row_of(t, srow);
    const uint32_t off = (uint32_t)row * (uint32_t)ROWB;
#pragma unroll
    for (int j = 0; j < NLD; ++j)  // (pieces past the row's end: its last piece again, not parked)
      st[j] = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)(off + (uint32_t)min(piece + j * LPR, NPC - 1) * 16u), 0, kAuxNontemporal);
    if constexpr (WK != 0) {
      if (piece == 0) sc = scale_of(row);
    }
  };
  // (the scales have four slots: a tile's are written a step before its multiply and read by the
  // emit waves a step after it, while the next tiles are already being parked)
  auto park = [&](const u32x4(&st)[NLD], float sc, int slot, int i) {
    unsigned char* dst = lds + slot * TILE + srow * PITCH;
#pragma unroll
    for (int j = 0; j < NLD; ++j) {
      const int pc = piece + j * LPR;
      if constexpr (WK == 0) {
        *reinterpret_cast<u32x4*>(dst + pc * 16) = st[j];
      } else {
        if (NPC % LPR == 0 || pc < NPC) {
          uint32_t o[8];
          codes_to_bf16<WK>(st[j], o);
          *reinterpret_cast<u32x4*>(dst + pc * 32) = u32x4{o[0], o[1], o[2], o[3]};
          *reinterpret_cast<u32x4*>(dst + pc * 32 + 16) = u32x4{o[4], o[5], o[6], o[7]};
        }
      }
    }
    if constexpr (WK != 0) {
      if (piece == 0) sc_sh[i & 3][srow] = sc;
    }
  };
  auto multiply = [&](int slot, int buf) {
    const unsigned char* src = lds + slot * TILE + ri * PITCH + (h * HS * 4 + kg) * 16;
    f32x4 acc{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < HS; ++s) acc = mfma_bf16(*reinterpret_cast<const u32x4*>(src + s * 64), qf[s], acc);
#pragma unroll
    for (int e = 0; e < 4; ++e) red[buf][h][nbw * 4 + e][lane] = acc[e];
  };
  u32x4 st0[NLD], st1[NLD];
  float sc0 = 1.f, sc1 = 1.f;
  load_stage(tile0, st0, sc0);
  load_stage(tile0 + 1, st1, sc1);
  __builtin_amdgcn_sched_barrier(0);
  park(st0, sc0, 0, 0);
  load_stage(tile0 + 2, st0, sc0);
  __builtin_amdgcn_sched_barrier(0);
  lds_barrier();
  for (int i = 0; i < ntiles; i += 2) {  // ntiles is even
    park(st1, sc1, 1, i + 1);
    __builtin_amdgcn_sched_barrier(0);
    load_stage(tile0 + i + 3, st1, sc1);
    __builtin_amdgcn_sched_barrier(0);
    multiply(0, 0);
    lds_barrier();
    park(st0, sc0, 0, i + 2);
    __builtin_amdgcn_sched_barrier(0);
    load_stage(tile0 + i + 4, st0, sc0);
    __builtin_amdgcn_sched_barrier(0);
    multiply(1, 1);
    lds_barrier();
  }
}

// --------------------------------------------------------------------------------- predict
template <int NB, int SPW, int NLW>
__global__ __launch_bounds__(kRowThreads) void predict_batch_kernel(const BatchParams P) {
  extern __shared__ __align__(16) float red_raw[];
  const int lane = threadIdx.x & (kWave - 1);
  const int ri = lane & 15, kg = lane >> 4;
  const int l = blockIdx.y;
  const int tiles_total = (P.d_ff + 15) / 16;
  const int tile0 = blockIdx.x * P.TPW1;
  if (tile0 >= tiles_total) return;
  float* S = P.S + (size_t)l * P.B * P.d_ff;
  float* ST = P.ST + (size_t)l * P.d_ff * P.BP;
  rows_times_tokens<NB, SPW, NLW, false>(
      static_cast<const bf16_t*>(P.k1n[l]), (uint32_t)P.d_ff * (uint32_t)P.r * 2u, P.r, P.q + (size_t)l * P.qslot, P.ldq, 0, P.B, tile0, P.TPW1,
      min(tile0 + P.TPW1, tiles_total), red_raw,
      [&](int t, int i) { return min(t * 16 + i, P.d_ff - 1); }, [](int, int, int) { return 0.f; },
      [&](int t, int nb, f32x4 v, f32x4) {
        const int b = nb * 16 + ri, j = t * 16 + 4 * kg;
        if (t >= tiles_total) return;
        if (b < P.B) {
          if ((P.d_ff & 3) == 0) {  // the four neurons of a lane are inside the layer together, or none is
            if (j < P.d_ff) *reinterpret_cast<f32x4*>(S + (size_t)b * P.d_ff + j) = v;
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (j + e < P.d_ff) S[(size_t)b * P.d_ff + j + e] = v[e];
          }
        }
        if (b < P.BP) {  // tokens past the batch have v = 0: whole lines are written
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (j + e < P.d_ff) ST[(size_t)(j + e) * P.BP + b] = v[e];
        }
      });
}

template <int WK, int NB, int CJ>
__global__ __launch_bounds__(staged_waves(NB, CJ) * kWave) void predict_staged_kernel(const BatchParams P) {
  extern __shared__ __align__(16) unsigned char staged_lds[];
  const int lane = threadIdx.x & (kWave - 1);
  const int ri = lane & 15, kg = lane >> 4;
  const int l = blockIdx.y;
  const int tiles_total = (P.d_ff + 15) / 16;
  const int tile0 = blockIdx.x * P.TPW1;
  if (tile0 >= tiles_total) return;
  float* S = P.S + (size_t)l * P.B * P.d_ff;
  float* ST = P.ST ? P.ST + (size_t)l * P.d_ff * P.BP : nullptr;  // (written only if a k2 kernel reads it)
  const float* k1s = reinterpret_cast<const float*>(static_cast<const char*>(P.k1n[l]) + (size_t)P.d_ff * P.r);  // (codes only)
  rows_times_tokens_staged<WK, NB, CJ, false>(
      P.k1n[l], (uint32_t)P.d_ff * (uint32_t)P.r * (WK ? 1u : 2u), P.q + (size_t)l * P.qslot, P.ldq, 0, P.B, tile0,
      P.TPW1, min(tile0 + P.TPW1, tiles_total), staged_lds,
      [&](int t, int i) { return min(t * 16 + i, P.d_ff - 1); }, [&](int row) { return k1s[row]; },
      [](int, int, int) { return 0.f; },
      [&](int t, int nb, f32x4 v, f32x4) {
        const int b = nb * 16 + ri, j = t * 16 + 4 * kg;
        if (t >= tiles_total) return;
        if (b < P.B) {
          if ((P.d_ff & 3) == 0) {  // the four neurons of a lane are inside the layer together, or none is
            if (j < P.d_ff) *reinterpret_cast<f32x4*>(S + (size_t)b * P.d_ff + j) = v;
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (j + e < P.d_ff) S[(size_t)b * P.d_ff + j + e] = v[e];
          }
        }
        if (ST != nullptr && b < P.BP) {  // tokens past the batch have v = 0: whole lines are written
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (j + e < P.d_ff) ST[(size_t)(j + e) * P.BP + b] = v[e];
        }
      });
}

// ------------------------------------------------------------------------ lane-crossing sums
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), c, false);
}
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_add(float x) {
  const int t = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, ROW_MASK, 0xf, false);
  return x + __int_as_float(t);
}
// Sum over the wavefront (quad swaps, row mirrors, row broadcasts), returned as a uniform value.
__device__ __forceinline__ float wave_total(float x) {
  x = dpp_add<0xB1, 0xf>(x);
  x = dpp_add<0x4E, 0xf>(x);
  x = dpp_add<0x141, 0xf>(x);
  x = dpp_add<0x140, 0xf>(x);
  x = dpp_add<0x142, 0xa>(x);
  x = dpp_add<0x143, 0xc>(x);
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}

// ---------------------------------------------------------------------------------- select
// One workgroup (4 waves) per (token, layer); the row of scores sits in registers (VPT per
// thread; small workgroups so that many rows are in flight per compute unit).
constexpr int kSelThreads = 256;
template <int VPT>
__global__ __launch_bounds__(kSelThreads) void select_batch_kernel(const BatchParams P) {
  constexpr int NWS = kSelThreads / kWave;
  __shared__ float red[NWS];
  __shared__ int wcount[NWS];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int b = blockIdx.x, l = blockIdx.y;
  const float* row = P.S + ((size_t)l * P.B + b) * P.d_ff;
  float v[VPT];
  float sum = 0.f;
#pragma unroll
  for (int k = 0; k < VPT; ++k) {
    const int j = tid + kSelThreads * k;
    v[k] = j < P.d_ff ? row[j] : 0.f;
  }
#pragma unroll
  for (int k = 0; k < VPT; ++k) sum += v[k];
  const float mean = block_sum<kSelThreads>(sum, red) / (float)P.d_ff;
  float sq = 0.f;
#pragma unroll
  for (int k = 0; k < VPT; ++k) {
    const float d = tid + kSelThreads * k < P.d_ff ? v[k] - mean : 0.f;
    sq += d * d;
  }
  const float m2 = block_sum<kSelThreads>(sq, red);
  const float theta = mean + sqrtf(m2 / (float)(P.d_ff - 1)) * P.z;
  if (tid == 0) {
    P.thetas[(size_t)l * P.B + b] = theta;
    if (P.theta) P.theta[(size_t)l * P.B + b] = theta;
  }
  int running = 0;
  const bool want_idx = P.idx || P.count;
#pragma unroll
  for (int k = 0; k < VPT; ++k) {
    if (kSelThreads * k >= P.d_ff) break;  // uniform
    const int j = tid + kSelThreads * k;
    const bool on = j < P.d_ff && v[k] > theta;
    const unsigned long long m = __ballot(on);
    if (lane == 0) P.tmask[((size_t)l * P.B + b) * kMaxWords + (j >> 6)] = m;
    if (want_idx) {
      __syncthreads();
      if (lane == 0) wcount[wave] = __popcll(m);
      __syncthreads();
      int before = 0, total = 0;
#pragma unroll
      for (int w = 0; w < NWS; ++w) {
        before += w < wave ? wcount[w] : 0;
        total += wcount[w];
      }
      if (on && P.idx) P.idx[((size_t)l * P.B + b) * P.d_ff + running + before + lanes_below(m)] = j;
      running += total;
    }
  }
  if (tid == 0 && P.count) P.count[(size_t)l * P.B + b] = running;
}

// One workgroup per layer: the union of the tokens' masks, word by word (plain stores and
// loads: no atomics, and nothing to clear beforehand), then the union's size and the neuron of
// every union rank in ascending order (prefix sums of the words' bit counts; a thread lists the
// bits of one 16-bit quarter of a word), which is what the k2 workgroups start from.
__global__ __launch_bounds__(4 * kMaxWords) void union_batch_kernel(const BatchParams P) {
  __shared__ unsigned long long part[4][kMaxWords];
  __shared__ int wprefix[kMaxWords + 1];
  __shared__ int wave_sum[kMaxWords / kWave];
  const int l = blockIdx.x, w = threadIdx.x % kMaxWords, q = threadIdx.x / kMaxWords;  // q: every 4th token
  const int lane = threadIdx.x & (kWave - 1);
  const bool live = w < (P.d_ff + 63) / 64;
  const unsigned long long* tm = P.tmask + (size_t)l * P.B * kMaxWords + w;
  unsigned long long m = 0ull;
  if (live) {
#pragma unroll 4
    for (int b = q; b < P.B; b += 4) m |= tm[(size_t)b * kMaxWords];
  }
  part[q][w] = m;
  __syncthreads();
  const unsigned long long word = part[0][w] | part[1][w] | part[2][w] | part[3][w];
  int inc = 0;
  if (q == 0) {  // the first kMaxWords threads: one word each, inclusive prefix sums inside each wave
    inc = __popcll(word);
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
      const int t = __shfl_up(inc, o, kWave);
      if (lane >= o) inc += t;
    }
    if (lane == kWave - 1) wave_sum[w / kWave] = inc;
  }
  __syncthreads();
  if (q == 0) {
    int before = 0;
#pragma unroll
    for (int i = 0; i < kMaxWords / kWave; ++i) before += i < w / kWave ? wave_sum[i] : 0;
    wprefix[w + 1] = before + inc;
    if (w == 0) wprefix[0] = 0;
  }
  __syncthreads();
  const int m_total = wprefix[kMaxWords];
  if (threadIdx.x == 0) {
    P.utotal[l] = m_total;
    if (P.ucount) P.ucount[l] = m_total;
  }
  unsigned bits = (unsigned)(word >> (16 * q)) & 0xffffu;
  int at = wprefix[w] + __popcll(word & ((1ull << (16 * q)) - 1ull));
  while (bits) {
    const int j = w * 64 + 16 * q + __builtin_ctz(bits);
    bits &= bits - 1;
    P.urow[(size_t)l * P.d_ff + at] = j;
    if (P.uidx) P.uidx[(size_t)l * P.d_ff + at] = j;
    ++at;
  }
}

// -------------------------------------------------------------------------------------- k2
// Shared opening of the k2 kernels: the union size and, in LDS, the neuron of every union rank
// the workgroup handles (ranks past the end repeat the last one).  Returns the union size;
// workgroups with no tile to do get -1.
template <int THREADS>
__device__ __forceinline__ int k2_ranks_to_rows(const BatchParams& P, int l, int tile0, int* rowidx) {
  const int m_total = P.utotal[l];
  const int tiles_total = (m_total + 15) / 16;
  if (tile0 >= tiles_total) return -1;
  const int32_t* urow = P.urow + (size_t)l * P.d_ff;
  for (int i = threadIdx.x; i < P.TPW2 * 16 + 16; i += THREADS) rowidx[i] = urow[min(tile0 * 16 + i, m_total - 1)];
  __syncthreads();
  return m_total;
}

// The activations of four consecutive union ranks of one token, u = GELU(s - theta) * g where
// the token activates the row and 0 elsewhere, as three bf16 planes.
__device__ __forceinline__ void k2_store_u(const BatchParams& P, uint16_t* up, int rho, int b, int m_total, float th,
                                           f32x4 g, f32x4 score) {
  float rest[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float a = score[e] - th;
    rest[e] = (rho + e < m_total && a > 0.f) ? gelu(a, P.gelu) * g[e] : 0.f;
  }
#pragma unroll
  for (int pl = 0; pl < kMaxPlanes; ++pl) {
    if (pl >= P.planes) break;
    const uint32_t w01 = pack_bf16x2_rne(rest[0], rest[1]), w23 = pack_bf16x2_rne(rest[2], rest[3]);
    rest[0] -= bf16_lo(w01);
    rest[1] -= bf16_hi(w01);
    rest[2] -= bf16_lo(w23);
    rest[3] -= bf16_hi(w23);
    *reinterpret_cast<u32x2*>(up + pl * P.plane + ((size_t)(rho >> 3) * P.B + b) * 8 + (rho & 7)) = u32x2{w01, w23};
  }
}

// Ranks between the last tile of the union and the end of the v phase's last 32-row group read
// as zero (called by the workgroup that holds the union's last tile).
template <int THREADS>
__device__ __forceinline__ void k2_zero_tail(const BatchParams& P, uint16_t* up, int from, int to) {
  for (int i = threadIdx.x; i < (to - from) * P.B; i += THREADS) {
    const int b = i / (to - from), rho = from + i % (to - from);
    for (int pl = 0; pl < P.planes; ++pl) up[pl * P.plane + ((size_t)(rho >> 3) * P.B + b) * 8 + (rho & 7)] = 0;
  }
}

template <int NB, int SPW, int NLW>
__global__ __launch_bounds__(kRowThreads) void k2_batch_kernel(const BatchParams P) {
  extern __shared__ __align__(16) float red_raw[];
  __shared__ int rowidx[32 * 16 + 16];
  const int tid = threadIdx.x, lane = tid & (kWave - 1);
  const int ri = lane & 15, kg = lane >> 4;
  const int l = blockIdx.y;
  const int tile0 = blockIdx.x * P.TPW2;
  const int m_total = k2_ranks_to_rows<kRowThreads>(P, l, tile0, rowidx);
  if (m_total < 0) return;
  const int tiles_total = (m_total + 15) / 16;
  const int rank_end = (m_total + 31) / 32 * 32;  // the v phase reads ranks below this
  const float* ST = P.ST + (size_t)l * P.d_ff * P.BP;
  float th[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) th[nb] = P.thetas[(size_t)l * P.B + min(nb * 16 + ri, P.B - 1)];
  uint16_t* up = P.up + (size_t)l * P.B * P.ldu;
  rows_times_tokens<NB, SPW, NLW, true>(
      static_cast<const bf16_t*>(P.k2n[l]), (uint32_t)P.d_ff * (uint32_t)(P.d_model - P.r) * 2u, P.d_model - P.r, P.q + (size_t)l * P.qslot, P.ldq,
      P.r, P.B, tile0, P.TPW2, min(tile0 + P.TPW2, tiles_total), red_raw,
      [&](int t, int i) { return rowidx[min((t - tile0) * 16 + i, P.TPW2 * 16 + 15)]; },
      [&](int t, int nb, int e) {  // the score the (row, token) pair will need
        const int b = min(nb * 16 + ri, P.B - 1);
        return ST[(size_t)rowidx[min((t - tile0) * 16 + 4 * kg + e, P.TPW2 * 16 + 15)] * P.BP + b];
      },
      [&](int t, int nb, f32x4 g, f32x4 score) {
        const int b = nb * 16 + ri;
        const int rho = t * 16 + 4 * kg;  // first of the lane's four ranks (inside one block of 8)
        if (b >= P.B || rho >= rank_end) return;
        k2_store_u(P, up, rho, b, m_total, th[nb], g, score);
      });
  if (tile0 + P.TPW2 >= tiles_total) k2_zero_tail<kRowThreads>(P, up, (tile0 + P.TPW2) * 16, rank_end);
}

template <int WK, int NB, int CJ>
__global__ __launch_bounds__(staged_waves(NB, CJ) * kWave) void k2_staged_kernel(const BatchParams P) {
  constexpr int THREADS = staged_waves(NB, CJ) * kWave;
  extern __shared__ __align__(16) unsigned char staged_lds[];
  __shared__ int rowidx[32 * 16 + 16];
  const int tid = threadIdx.x, lane = tid & (kWave - 1);
  const int ri = lane & 15, kg = lane >> 4;
  const int l = blockIdx.y;
  const int tile0 = blockIdx.x * P.TPW2;
  const int m_total = k2_ranks_to_rows<THREADS>(P, l, tile0, rowidx);
  if (m_total < 0) return;
  const int tiles_total = (m_total + 15) / 16;
  const int rank_end = (m_total + 31) / 32 * 32;  // the v phase reads ranks below this
  const float* S = P.S + (size_t)l * P.B * P.d_ff;
  float th[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) th[nb] = P.thetas[(size_t)l * P.B + min(nb * 16 + ri, P.B - 1)];
  uint16_t* up = P.up + (size_t)l * P.B * P.ldu;
  // (codes: a row's two scales travel as their product; the V step then multiplies plain codes)
  const float* k2s = reinterpret_cast<const float*>(static_cast<const char*>(P.k2n[l]) + (size_t)P.d_ff * (P.d_model - P.r));
  const float* vs = reinterpret_cast<const float*>(static_cast<const char*>(P.vn[l]) + (size_t)P.d_ff * P.d_model);
  rows_times_tokens_staged<WK, NB, CJ, true>(
      P.k2n[l], (uint32_t)P.d_ff * (uint32_t)(P.d_model - P.r) * (WK ? 1u : 2u), P.q + (size_t)l * P.qslot, P.ldq,
      P.r, P.B, tile0, P.TPW2, min(tile0 + P.TPW2, tiles_total), staged_lds,
      [&](int t, int i) { return rowidx[min((t - tile0) * 16 + i, P.TPW2 * 16 + 15)]; },
      [&](int row) { return k2s[row] * vs[row]; },
      [&](int t, int nb, int e) {  // the score the (row, token) pair will need, from the token-major array
        const int b = min(nb * 16 + ri, P.B - 1);
        return S[(size_t)b * P.d_ff + rowidx[min((t - tile0) * 16 + 4 * kg + e, P.TPW2 * 16 + 15)]];
      },
      [&](int t, int nb, f32x4 g, f32x4 score) {
        const int b = nb * 16 + ri;
        const int rho = t * 16 + 4 * kg;  // first of the lane's four ranks (inside one block of 8)
        if (b >= P.B || rho >= rank_end) return;
        k2_store_u(P, up, rho, b, m_total, th[nb], g, score);
      });
  if (tile0 + P.TPW2 >= tiles_total) k2_zero_tail<THREADS>(P, up, (tile0 + P.TPW2) * 16, rank_end);
}

// ------------------------------------------------------- rows x tokens, whole rows (<= 16 tokens)
// The k-split kernels above read a row in 64-byte pieces (the shape the 16x16x32 operand asks
// for), which the memory system serves at some 85 % of what whole rows reach.  Here a wave
// takes FOUR CONSECUTIVE ROWS per step and reads them whole: lane (block = lane / 4, i = lane % 4)
// loads the 16-byte chunks block + 16 c, c < CH, of row i, so one load instruction covers 256
// contiguous bytes of each of four rows (K = 128 CH).  The products run on the 4x4x4 matrix
// instruction, whose 16 independent blocks are exactly this layout: block b multiplies rows
// i < 4 by tokens j < 4 over four k values, A[i][k] in lane 4 b + i, B[k][j] in lane 4 b + j,
// D[i][j] in lane 4 b + j, register i.  A chunk (8 k values) feeds two instructions per group of
// four tokens; the token operands sit in LDS in lane order.  After the row's last chunk the 16
// blocks hold partial sums over disjoint k ranges: they are added across lanes, halving the
// number of live values at each stage, so that lane (b, j) ends with the sum for row b % 4 and
// token 4 (b / 4) + j, which goes to LDS; the workgroup stores everything after its last step
// (no store between the loads: they share the loads' counter).  Two steps are in flight per wave.
constexpr int kR4Threads = 256;
typedef short s16x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ f32x4 mfma_4x4x4(uint32_t a0, uint32_t a1, uint32_t b0, uint32_t b1, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(__builtin_bit_cast(s16x4_t, u32x2{a0, a1}),
                                                __builtin_bit_cast(s16x4_t, u32x2{b0, b1}), c, 0, 0, 0);
}
// Halves of the wavefront (rows of 16 lanes) trade places: after the call and the addition the
// lanes whose bit 5 (bit 4) is clear hold `lo` summed over that bit, the others hold `hi`.
__device__ __forceinline__ float fold_bit5(float lo, float hi) {
  const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(lo), __float_as_uint(hi), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float fold_bit4(float lo, float hi) {
  const u32x2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(lo), __float_as_uint(hi), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
template <int NG>
__device__ __forceinline__ float blocks_to_lanes(const f32x4 (&acc)[NG], int lane) {
  float v[16];
#pragma unroll
  for (int n = 0; n < 16; ++n) v[n] = n / 4 < NG ? acc[n / 4 < NG ? n / 4 : 0][n % 4] : 0.f;
  float w8[8], w4[4];
#pragma unroll
  for (int n = 0; n < 8; ++n) w8[n] = fold_bit5(v[n], v[n + 8]);
#pragma unroll
  for (int n = 0; n < 4; ++n) w4[n] = fold_bit4(w8[n], w8[n + 4]);
#pragma unroll
  for (int n = 0; n < 4; ++n) {  // the four blocks of a row of 16 lanes: rotations by 4 and 8
    w4[n] = dpp_add<0x124, 0xf>(w4[n]);
    w4[n] = dpp_add<0x128, 0xf>(w4[n]);
  }
  const int sel = (lane >> 2) & 3;
  return sel == 0 ? w4[0] : sel == 1 ? w4[1] : sel == 2 ? w4[2] : w4[3];
}

constexpr int r4_pitch(int NS) { return NS * 16 + 4; }  // floats between tokens of the result tile in LDS

// row_of(local row) gives the matrix row of the workgroup's local row (any valid row for rows
// that do not count); rows from `nrows` on are not read when a whole step lies past them.
// A row is CH pieces of 256 bytes per block column: 128 CH bf16 elements or 256 CH codes.
template <int WK, int NG, int CH, int NS, typename RowOf>
__device__ __forceinline__ void rows4_sweep(const void* __restrict__ w, uint32_t w_bytes,
                                            const bf16_t* __restrict__ q, int64_t ldq, int qoff, int B, int nrows,
                                            u32x4* qsh, RowOf row_of, float* out) {
  constexpr int TPP = WK ? 2 : 1;  // 16-byte token operands per weight piece (8 or 16 elements of k)
  const int tid = threadIdx.x, lane = tid & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int blk = lane >> 2, i4 = lane & 3;
  // token operands in lane order: entry ((c NG + g) TPP + h) 64 + lane = elements
  // 8 (TPP (blk + 16 c) + h) .. + 7 of token 4 g + i4
  auto stage_tokens = [&]() {
    for (int e = tid; e < CH * NG * TPP * kWave; e += kR4Threads) {
      const int ln = e & (kWave - 1), cgh = e >> 6, h = cgh % TPP, cg = cgh / TPP, g = cg % NG, c = cg / NG;
      const int t = 4 * g + (ln & 3), ch = TPP * ((ln >> 2) + 16 * c) + h;
      u32x4 v{0u, 0u, 0u, 0u};
      if (t < B) v = ld16(q + (int64_t)t * ldq + qoff + ch * 8);
      qsh[e] = v;
    }
    __syncthreads();
  };
  auto load_step = [&](int s, u32x4(&a)[CH]) {
    const int lr = s * 16 + wave * 4;  // steps past the rows: a descriptor without records
    const __amdgpu_buffer_rsrc_t rs =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(w), 0, lr < nrows ? (int)w_bytes : 0, 0x00020000);
    const uint32_t off = (uint32_t)row_of(lr + i4) * (uint32_t)(CH * 256) + (uint32_t)blk * 16u;
#pragma unroll
    for (int c = 0; c < CH; ++c) a[c] = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)(off + (uint32_t)c * 256u), 0, kAuxNontemporal);
  };
  auto multiply = [&](const u32x4(&a)[CH], int s) {
    f32x4 acc[NG];
#pragma unroll
    for (int g = 0; g < NG; ++g) acc[g] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      if constexpr (WK == 0) {
#pragma unroll
        for (int g = 0; g < NG; ++g) {
          const u32x4 t = qsh[(c * NG + g) * kWave + lane];
          acc[g] = mfma_4x4x4(a[c][0], a[c][1], t[0], t[1], acc[g]);
          acc[g] = mfma_4x4x4(a[c][2], a[c][3], t[2], t[3], acc[g]);
        }
      } else {
        uint32_t o[8];
        codes_to_bf16<WK>(a[c], o);
#pragma unroll
        for (int g = 0; g < NG; ++g)
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            const u32x4 t = qsh[((c * NG + g) * 2 + h) * kWave + lane];
            acc[g] = mfma_4x4x4(o[4 * h], o[4 * h + 1], t[0], t[1], acc[g]);
            acc[g] = mfma_4x4x4(o[4 * h + 2], o[4 * h + 3], t[2], t[3], acc[g]);
          }
      }
    }
    const float val = blocks_to_lanes<NG>(acc, lane);
    if ((blk >> 2) < NG) out[(4 * (blk >> 2) + i4) * r4_pitch(NS) + s * 16 + wave * 4 + (blk & 3)] = val;
  };
  u32x4 a0[CH], a1[CH];
  if constexpr (NS > 4) stage_tokens();
  load_step(0, a0);
  load_step(1, a1);
  __builtin_amdgcn_sched_barrier(0);
  if constexpr (NS <= 4) stage_tokens();
#pragma unroll
  for (int s = 0; s < NS; s += 2) {
    multiply(a0, s);
    __builtin_amdgcn_sched_barrier(0);
    if (s + 2 < NS) load_step(s + 2, a0);
    __builtin_amdgcn_sched_barrier(0);
    multiply(a1, s + 1);
    __builtin_amdgcn_sched_barrier(0);
    if (s + 3 < NS) load_step(s + 3, a1);
    __builtin_amdgcn_sched_barrier(0);
  }
  __syncthreads();
}

// Rows of one weight array in bytes and, for codes, the fp32 scales that follow the last row.
template <int WK, int CH>
__device__ __forceinline__ const float* r4_scales(const void* w, int rows) {
  if constexpr (WK != 0) return reinterpret_cast<const float*>(static_cast<const char*>(w) + (size_t)rows * (CH * 256));
  else return nullptr;
}

template <int WK, int NG, int CH, int NS>
__global__ __launch_bounds__(kR4Threads) void predict_rows4_kernel(const BatchParams P) {
  extern __shared__ __align__(16) u32x4 qsh[];
  constexpr int RW = NS * 16, PITCH = r4_pitch(NS);
  __shared__ __align__(16) float s_sh[4 * NG * PITCH];
  const int l = blockIdx.y;
  const int row0 = blockIdx.x * RW, nrows = min(RW, P.d_ff - row0);
  if (nrows <= 0) return;
  rows4_sweep<WK, NG, CH, NS>(P.k1n[l], (uint32_t)P.d_ff * (uint32_t)(CH * 256), P.q + (size_t)l * P.qslot, P.ldq, 0, P.B,
                              nrows, qsh, [&](int lr) { return min(row0 + lr, P.d_ff - 1); }, s_sh);
  const float* scales = r4_scales<WK, CH>(P.k1n[l], P.d_ff);
  float* S = P.S + (size_t)l * P.B * P.d_ff;
  for (int idx = threadIdx.x; idx < P.B * RW; idx += kR4Threads) {
    const int t = idx / RW, rr = idx % RW;
    if (rr < nrows) {
      float v = s_sh[t * PITCH + rr];
      if constexpr (WK != 0) v *= scales[row0 + rr];
      S[(size_t)t * P.d_ff + row0 + rr] = v;
    }
  }
  if (P.ST == nullptr) return;  // (the whole-row k2 kernel reads the token-major scores)
  float* ST = P.ST + (size_t)l * P.d_ff * P.BP;
  for (int idx = threadIdx.x; idx < RW * P.BP; idx += kR4Threads) {  // tokens past the batch: zeros (whole lines)
    const int rr = idx / P.BP, t = idx % P.BP;
    if (rr < nrows) {
      float v = t < P.B ? s_sh[t * PITCH + rr] : 0.f;
      if constexpr (WK != 0) v *= scales[row0 + rr];
      ST[(size_t)(row0 + rr) * P.BP + t] = v;
    }
  }
}

template <int WK, int NG, int CH, int NS>
__global__ __launch_bounds__(kR4Threads) void k2_rows4_kernel(const BatchParams P) {
  extern __shared__ __align__(16) u32x4 qsh[];
  constexpr int RW = NS * 16, PITCH = r4_pitch(NS), IT = NS / 4;
  static_assert(NS % 4 == 0, "a pass of the closing loop covers 64 ranks");
  __shared__ int rowidx[RW + 16];
  __shared__ __align__(16) float g_sh[4 * NG * PITCH];
  const int tid = threadIdx.x;
  const int l = blockIdx.y;
  const int tile0 = blockIdx.x * P.TPW2;  // the launch sets TPW2 = NS
  const int m_total = k2_ranks_to_rows<kR4Threads>(P, l, tile0, rowidx);
  if (m_total < 0) return;
  const int tiles_total = (m_total + 15) / 16;
  const int rank_end = (m_total + 31) / 32 * 32;  // the v phase reads ranks below this
  const int rank0 = tile0 * 16;
  // closing work item m of a thread: token b, ranks rank0 + 4 rq ..+3; its scores are asked for
  // ahead of the weight rows, from the token-major array (the union's rows ascend, so the four
  // of an item, and the items of a token, lie close together in the token's row of scores)
  const int b = tid & 15;
  const float* Sb = P.S + ((size_t)l * P.B + min(b, P.B - 1)) * P.d_ff;
  f32x4 score[IT], scale[IT];
  // (codes: the row's two scales travel as their product, which is all the sum needs:
  // u_j Vn[j] = GELU(a) (scale_k2 g) (scale_v codes); the V step then multiplies plain codes)
  const float* k2s = r4_scales<WK, CH>(P.k2n[l], P.d_ff);
  const float* vs = WK != 0 ? reinterpret_cast<const float*>(static_cast<const char*>(P.vn[l]) + (size_t)P.d_ff * P.d_model) : nullptr;
#pragma unroll
  for (int m = 0; m < IT; ++m)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int j = rowidx[((tid >> 4) + 16 * m) * 4 + e];
      score[m][e] = Sb[j];
      if constexpr (WK != 0) scale[m][e] = k2s[j] * vs[j];
      else scale[m][e] = 1.f;
    }
  const float th = P.thetas[(size_t)l * P.B + min(b, P.B - 1)];
  rows4_sweep<WK, NG, CH, NS>(P.k2n[l], (uint32_t)P.d_ff * (uint32_t)(CH * 256), P.q + (size_t)l * P.qslot, P.ldq, P.r, P.B,
                              m_total - rank0, qsh, [&](int lr) { return rowidx[lr]; }, g_sh);
  uint16_t* up = P.up + (size_t)l * P.B * P.ldu;
#pragma unroll
  for (int m = 0; m < IT; ++m) {
    const int rq = (tid >> 4) + 16 * m, rho = rank0 + 4 * rq;
    if (b < P.B && rho < rank_end) {
      f32x4 g = *reinterpret_cast<const f32x4*>(&g_sh[b * PITCH + 4 * rq]);
      if constexpr (WK != 0) g *= scale[m];
      k2_store_u(P, up, rho, b, m_total, th, g, score[m]);
    }
  }
  if (tile0 + NS >= tiles_total) k2_zero_tail<kR4Threads>(P, up, (tile0 + NS) * 16, rank_end);
}

// --------------------------------------------------------------------------------------- v
// Workgroup = NWV waves (4..8) x 64 columns, one slice of the union's 32-row groups.  Per
// group a wave loads 32 rows x 128 bytes (lane = row 8 t + lane / 8, 16-byte chunk lane % 8,
// t < 4), parks them in its own LDS tile with row 8 t + j at position 4 j + t (pitch 160 bytes:
// the four lane groups of a transposed read then hit disjoint banks), and reads back, per
// 16-column tile, the 8 rows 8 kg + e of column ri as the B operand.  The A operands (8
// consecutive ranks of token ri from each bf16 plane of u) are the same for every wave: the
// workgroup fetches them once per group into LDS, already in lane order.  One barrier per
// group; the next group's rows and activations are in flight during the MFMAs.
constexpr int kVMinWaves = 4, kVMaxWaves = 8;
template <int NB, int WK = 0>
__global__ __launch_bounds__(kVMaxWaves * kWave, (NB == 4 ? 2 : NB == 3 ? 3 : 4)) void v_batch_kernel(const BatchParams P) {
  // WK != 0: Vn holds 8-bit codes (the rows' scales are already inside u).  A wave's 64 columns
  // are then 64 bytes of a row: lane = (row lane / 4 of 16, 16-byte piece lane % 4), two loads
  // per 32-row group; the codes are widened to bf16 when the rows are parked in LDS, and the
  // rest of the kernel is the same.
  constexpr int NLV = WK ? 2 : 4;  // row loads per lane and group
  // (with four token blocks a wave keeps two groups in flight: measured 5 % on the call there,
  // nothing or a loss with fewer, where more workgroups share a compute unit)
  constexpr bool DEEP = NB == 4;
  constexpr int kPlanes = planes_for(NB);
  constexpr int UCH = kPlanes * NB * kWave;                            // 16-byte chunks of u per group
  constexpr int MINW = NB >= 3 ? 6 : kVMinWaves;                        // fewest waves the launch uses
  constexpr int UPT = (UCH + MINW * kWave - 1) / (MINW * kWave);        // most chunks per thread
  extern __shared__ __align__(16) unsigned char lds[];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), nthreads = blockDim.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int nwv = nthreads / kWave;
  unsigned char* mine = lds + (size_t)wave * 32 * kVPitch;
  u32x4* ush = reinterpret_cast<u32x4*>(lds + (size_t)nwv * 32 * kVPitch);  // [2][UCH]
  const int ri = lane & 15, kg = lane >> 4;
  // Workgroup -> (column slab, row slice, layer).  The slabs of one (slice, layer) read the same
  // activations; workgroups are dealt to the eight dies in turn, each with an L2 of its own, so
  // the launch order is folded: die d takes the d-th eighth of the (layer, slice, slab) list,
  // slab fastest, and the slabs that share activations meet in one L2 at about the same time
  // (dealt in launch order they sat on different dies and each fetched its own copy).
  const int total = P.VSLABS * P.KS * P.n_layers, per_die = (total + 7) / 8;
  const int m = (int)(blockIdx.x & 7u) * per_die + (int)(blockIdx.x >> 3);
  if (m >= total) return;
  const int slab = m % P.VSLABS, ks = (m / P.VSLABS) % P.KS, l = m / (P.VSLABS * P.KS);
  const int col_own = (slab * nwv + wave) * 64;
  // a wave past the last column still helps with u and the barriers; its row loads go to the
  // last strip (unconditional loads keep the number in flight a compile-time constant)
  const bool active = col_own < P.d_model;
  const int col0 = active ? col_own : P.d_model - 64;
  const int m_total = P.utotal[l];
  const int groups_total = (m_total + 31) / 32;
  const int per = (groups_total + P.KS - 1) / P.KS;
  const int g0 = ks * per, g1 = min(g0 + per, groups_total);
  const char* vn = static_cast<const char*>(P.vn[l]);
  const int32_t* urow = P.urow + (size_t)l * P.d_ff;
  const uint16_t* up = P.up + (size_t)l * P.B * P.ldu;

  f32x4 acc[4][NB];
#pragma unroll
  for (int ct = 0; ct < 4; ++ct)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[ct][nb] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int lr = lane >> 3, lc = lane & 7;
  // neuron of rank 32 g + lane % 32 (ranks past the end repeat the last neuron; their u is 0)
  auto load_idx = [&](int g) { return urow[max(0, min(g * 32 + (lane & 31), m_total - 1))]; };
  auto load_rows = [&](int jn, u32x4(&v)[NLV]) {
#pragma unroll
    for (int t = 0; t < NLV; ++t) {
      if constexpr (WK == 0) {
        const int j = __shfl(jn, 8 * t + lr, kWave);
        v[t] = ld16_stream(vn + ((int64_t)j * P.d_model + col0 + lc * 8) * 2);
      } else {
        const int j = __shfl(jn, 16 * t + (lane >> 2), kWave);
        v[t] = ld16_stream(vn + (int64_t)j * P.d_model + col0 + (lane & 3) * 16);
      }
    }
  };
  // parks the group's rows in the wave's LDS tile: row 8 t + j at position 4 j + t
  auto park_rows = [&](const u32x4(&v)[NLV]) {
#pragma unroll
    for (int t = 0; t < NLV; ++t) {
      if constexpr (WK == 0) {
        *reinterpret_cast<u32x4*>(mine + (4 * lr + t) * kVPitch + lc * 16) = v[t];
      } else {
        const int row = 16 * t + (lane >> 2);
        uint32_t o[8];
        codes_to_bf16<WK>(v[t], o);
        unsigned char* dst = mine + (4 * (row & 7) + (row >> 3)) * kVPitch + (lane & 3) * 32;
        *reinterpret_cast<u32x4*>(dst) = u32x4{o[0], o[1], o[2], o[3]};
        *reinterpret_cast<u32x4*>(dst + 16) = u32x4{o[4], o[5], o[6], o[7]};
      }
    }
  };
  auto load_u = [&](int g, u32x4(&a)[UPT]) {
#pragma unroll
    for (int i = 0; i < UPT; ++i) {
      const int c = tid + i * nthreads;
      if (c < UCH) {
        const int cl = c & (kWave - 1), nb = (c >> 6) % NB, pl = (c >> 6) / NB;
        const int b = nb * 16 + (cl & 15);
        // tokens past the batch re-read the last token; they are zeroed when the chunk is parked
        // in LDS (a select here would have to wait for the load, and with it for every load
        // issued before it)
        a[i] = ld16(up + pl * P.plane + ((size_t)(g * 4 + (cl >> 4)) * P.B + min(b, P.B - 1)) * 8);
      }
    }
  };
  bool u_pad[UPT];
#pragma unroll
  for (int i = 0; i < UPT; ++i) {
    const int c = tid + i * nthreads;
    u_pad[i] = ((c >> 6) % NB) * 16 + (c & 15) >= P.B;
  }
  if constexpr (DEEP) {
   if (g0 < g1) {
    // Two groups are in flight per wave (two register sets, alternating in an unrolled pair of
    // steps).  A step parks its group in LDS, requests the group two ahead into the registers
    // it has just emptied (rows, then activations, then the row indices of the group four
    // ahead: loads return in order, so each is asked for after everything that is needed
    // before it), and multiplies after the barrier.  Groups past the slice's last are the last
    // one fetched again; their multiply is skipped.
    const int last = g1 - 1;
    auto step = [&](int g, u32x4(&v)[NLV], u32x4(&ur)[UPT], int& jn) {
      u32x4* ub = ush + ((g - g0) & 1) * UCH;
      if (active) park_rows(v);
#pragma unroll
      for (int i = 0; i < UPT; ++i)
        if (tid + i * nthreads < UCH) ub[tid + i * nthreads] = u_pad[i] ? u32x4{0u, 0u, 0u, 0u} : ur[i];
      load_rows(jn, v);
      load_u(min(g + 2, last), ur);
      jn = load_idx(min(g + 4, last));
      lds_barrier();
      if (active && g <= last) {
        u32x4 af[NB][kPlanes];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
          for (int pl = 0; pl < kPlanes; ++pl) af[nb][pl] = ub[(pl * NB + nb) * kWave + lane];
#pragma unroll
        for (int ct = 0; ct < 4; ++ct) {
          u32x4 bv;
#pragma unroll
          for (int e = 0; e < 8; e += 2) {
            const uint32_t x0 = *reinterpret_cast<const uint16_t*>(mine + (4 * e + kg) * kVPitch + (ct * 16 + ri) * 2);
            const uint32_t x1 = *reinterpret_cast<const uint16_t*>(mine + (4 * (e + 1) + kg) * kVPitch + (ct * 16 + ri) * 2);
            bv[e >> 1] = x0 | (x1 << 16);
          }
#pragma unroll
          for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int pl = kPlanes - 1; pl >= 0; --pl) acc[ct][nb] = mfma_bf16(af[nb][pl], bv, acc[ct][nb]);
        }
      }
    };
    u32x4 v0[NLV], v1[NLV], ur0[UPT], ur1[UPT];
    int jn0 = load_idx(g0), jn1 = load_idx(min(g0 + 1, last));
    load_rows(jn0, v0);
    load_u(g0, ur0);
    load_rows(jn1, v1);
    load_u(min(g0 + 1, last), ur1);
    jn0 = load_idx(min(g0 + 2, last));
    jn1 = load_idx(min(g0 + 3, last));
    for (int g = g0; g < g1; g += 2) {
      step(g, v0, ur0, jn0);
      step(g + 1, v1, ur1, jn1);
    }
   }
  } else
  if (g0 < g1) {
    u32x4 v0[NLV], ur[UPT];
    int jn = load_idx(g0);
    load_rows(jn, v0);
    load_u(g0, ur);
    jn = load_idx(min(g0 + 1, g1 - 1));
    for (int g = g0; g < g1; ++g) {
      u32x4* ub = ush + ((g - g0) & 1) * UCH;
      if (active) park_rows(v0);
#pragma unroll
      for (int i = 0; i < UPT; ++i)
        if (tid + i * nthreads < UCH) ub[tid + i * nthreads] = u_pad[i] ? u32x4{0u, 0u, 0u, 0u} : ur[i];
      // the row indices two groups ahead are requested first (loads return in order: waiting
      // for them in the next round must not mean waiting for that round's rows), then the rows
      // and activations of the next group (the last group is simply fetched again)
      const int jn2 = load_idx(min(g + 2, g1 - 1));
      load_rows(jn, v0);
      load_u(min(g + 1, g1 - 1), ur);
      jn = jn2;
      lds_barrier();
      if (active) {
        u32x4 af[NB][kPlanes];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
          for (int pl = 0; pl < kPlanes; ++pl) af[nb][pl] = ub[(pl * NB + nb) * kWave + lane];
#pragma unroll
        for (int ct = 0; ct < 4; ++ct) {
          u32x4 bv;
#pragma unroll
          for (int e = 0; e < 8; e += 2) {
            const uint32_t x0 = *reinterpret_cast<const uint16_t*>(mine + (4 * e + kg) * kVPitch + (ct * 16 + ri) * 2);
            const uint32_t x1 = *reinterpret_cast<const uint16_t*>(mine + (4 * (e + 1) + kg) * kVPitch + (ct * 16 + ri) * 2);
            bv[e >> 1] = x0 | (x1 << 16);
          }
#pragma unroll
          for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int pl = kPlanes - 1; pl >= 0; --pl) acc[ct][nb] = mfma_bf16(af[nb][pl], bv, acc[ct][nb]);
        }
      }
    }
  }
  if (!active) return;
  // D[token 4 kg + e][column ri] of every (column tile, token block)
  float* dst = P.part + ((size_t)l * P.KS + ks) * P.B * P.d_model;
#pragma unroll
  for (int ct = 0; ct < 4; ++ct)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int b = nb * 16 + 4 * kg + e;
        if (b < P.B) dst[(size_t)b * P.d_model + col0 + ct * 16 + ri] = acc[ct][nb][e];
      }
}

// ---------------------------------------------------------------------------------- reduce
__global__ __launch_bounds__(256) void reduce_batch_kernel(const BatchParams P) {
  const int l = blockIdx.y;
  const size_t n = (size_t)P.B * P.d_model;
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const float* p = P.part + (size_t)l * P.KS * n + i;
  float acc = 0.f;
  for (int ks = 0; ks < P.KS; ++ks) acc += p[(size_t)ks * n];
  P.y[(size_t)l * n + i] = acc;
}

size_t align256(size_t v) { return (v + 255) / 256 * 256; }

// Waves of a v workgroup: the largest count in 4..8 that divides the 64-column strips evenly.
// (at least 6 for more than 32 tokens, so that a thread fetches at most two chunks of u per group)
int v_waves(int d_model, int nb) {
  const int n64 = (d_model + 63) / 64, lo = nb >= 3 ? 6 : kVMinWaves;
  for (int w = kVMaxWaves; w >= lo; --w)
    if (n64 % w == 0) return w;
  return n64 < lo ? lo : kVMaxWaves;
}
int v_slabs(int d_model, int nb) { return ((d_model + 63) / 64 + v_waves(d_model, nb) - 1) / v_waves(d_model, nb); }
int part_rows(int d_model) { return kBatchMaxLayers + (768 + v_slabs(d_model, 4) - 1) / v_slabs(d_model, 4); }

struct BatchLayout {
  size_t S, ST, thetas, tmask, urow, utotal, up, plane, part, total;
  int ldu;
};

BatchLayout batch_layout(int d_model, int d_ff, int B) {
  BatchLayout s;
  const size_t L = kBatchMaxLayers;
  s.ldu = (d_ff + 64 + 7) / 8 * 8;
  size_t o = 0;
  s.S = o;      o += align256(L * B * (size_t)d_ff * 4);
  s.ST = o;     o += align256(L * (size_t)((B + 15) / 16 * 16) * (size_t)d_ff * 4);
  s.thetas = o; o += align256(L * B * 4);
  s.tmask = o;  o += align256(L * B * kMaxWords * 8);
  s.urow = o;   o += align256(L * (size_t)d_ff * 4);
  s.utotal = o; o += align256(L * 4);
  s.plane = align256(L * B * (size_t)s.ldu * 2) / 2;
  s.up = o;     o += kMaxPlanes * s.plane * 2;
  s.part = o;   o += align256((size_t)part_rows(d_model) * B * (size_t)d_model * 4);
  s.total = o;
  return s;
}

// Loader waves and k steps per loader for a row of K elements: the smallest (NLW, SPW) whose
// NLW * SPW steps of 32 cover K.  Returns false when none of the compiled ones does.
bool split_for(int K, int* nlw, int* spw) {
  static const int cand[][2] = {{8, 4}, {10, 4}, {8, 6}, {10, 6}, {8, 8}};
  for (const auto& c : cand)
    if (c[0] * c[1] * 32 >= K) {
      *nlw = c[0];
      *spw = c[1];
      return true;
    }
  return false;
}

template <int NB, int SPW, int NLW>
hipError_t launch_rows(const BatchParams& P, int mode, dim3 grid, hipStream_t st) {
  const size_t dyn = rows_lds_bytes<NB>();
  const void* kern = mode == 0 ? reinterpret_cast<const void*>(predict_batch_kernel<NB, SPW, NLW>)
                               : reinterpret_cast<const void*>(k2_batch_kernel<NB, SPW, NLW>);
  const hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn);
  if (e != hipSuccess) return e;
  if (mode == 0) hipLaunchKernelGGL((predict_batch_kernel<NB, SPW, NLW>), grid, dim3(kRowThreads), dyn, st, P);
  else hipLaunchKernelGGL((k2_batch_kernel<NB, SPW, NLW>), grid, dim3(kRowThreads), dyn, st, P);
  return hipGetLastError();
}
template <int NB>
hipError_t launch_rows_split(const BatchParams& P, int mode, int nlw, int spw, dim3 grid, hipStream_t st) {
  if (nlw == 8 && spw == 4) return launch_rows<NB, 4, 8>(P, mode, grid, st);
  if (nlw == 10 && spw == 4) return launch_rows<NB, 4, 10>(P, mode, grid, st);
  if (nlw == 8 && spw == 6) return launch_rows<NB, 6, 8>(P, mode, grid, st);
  if (nlw == 10 && spw == 6) return launch_rows<NB, 6, 10>(P, mode, grid, st);
  if (nlw == 8 && spw == 8) return launch_rows<NB, 8, 8>(P, mode, grid, st);
  return hipErrorInvalidValue;
}
hipError_t launch_rows_nb(const BatchParams& P, int mode, int nb, int K, dim3 grid, hipStream_t st) {
  int nlw = 0, spw = 0;
  if (!split_for(K, &nlw, &spw)) return hipErrorInvalidValue;
  switch (nb) {
    case 1: return launch_rows_split<1>(P, mode, nlw, spw, grid, st);
    case 2: return launch_rows_split<2>(P, mode, nlw, spw, grid, st);
    case 3: return launch_rows_split<3>(P, mode, nlw, spw, grid, st);
    case 4: return launch_rows_split<4>(P, mode, nlw, spw, grid, st);
    default: return hipErrorInvalidValue;
  }
}

// Staged kernels: rows of K = 256 CJ elements for the compiled CJ (a compute wave keeps the token
// operands of its part of a row in registers: 128 of them would be needed for rows of 2048
// elements with more than two token blocks).
int staged_cj(int K, int nb) {
  if (K % 256 != 0) return 0;
  const int cj = K / 256;
  return ((cj >= 2 && cj <= 6) || (cj == 8 && nb <= 2)) ? cj : 0;
}
template <int WK, int NB, int CJ>
hipError_t launch_staged(const BatchParams& P, int mode, dim3 grid, hipStream_t st) {
  const size_t dyn = staged_lds_bytes<NB, CJ>();
  const void* kern = mode == 0 ? reinterpret_cast<const void*>(predict_staged_kernel<WK, NB, CJ>)
                               : reinterpret_cast<const void*>(k2_staged_kernel<WK, NB, CJ>);
  const hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn);
  if (e != hipSuccess) return e;
  if (mode == 0) hipLaunchKernelGGL((predict_staged_kernel<WK, NB, CJ>), grid, dim3(staged_waves(NB, CJ) * kWave), dyn, st, P);
  else hipLaunchKernelGGL((k2_staged_kernel<WK, NB, CJ>), grid, dim3(staged_waves(NB, CJ) * kWave), dyn, st, P);
  return hipGetLastError();
}
template <int WK, int NB>
hipError_t launch_staged_cj(const BatchParams& P, int mode, int cj, dim3 grid, hipStream_t st) {
  switch (cj) {
    case 2: return launch_staged<WK, NB, 2>(P, mode, grid, st);
    case 3: return launch_staged<WK, NB, 3>(P, mode, grid, st);
    case 4: return launch_staged<WK, NB, 4>(P, mode, grid, st);
    case 5: return launch_staged<WK, NB, 5>(P, mode, grid, st);
    case 6: return launch_staged<WK, NB, 6>(P, mode, grid, st);
    case 8: if constexpr (NB <= 2) return launch_staged<WK, NB, 8>(P, mode, grid, st); else return hipErrorInvalidValue;
    default: return hipErrorInvalidValue;
  }
}
// (three token blocks run as four: the fourth block's operands are zeros)
template <int WK>
hipError_t launch_staged_nb(const BatchParams& P, int mode, int nb, int cj, dim3 grid, hipStream_t st) {
  return nb == 1 ? launch_staged_cj<WK, 1>(P, mode, cj, grid, st)
         : nb == 2 ? launch_staged_cj<WK, 2>(P, mode, cj, grid, st)
                   : launch_staged_cj<WK, 4>(P, mode, cj, grid, st);
}
hipError_t launch_staged_wk(const BatchParams& P, int wkind, int mode, int nb, int cj, dim3 grid, hipStream_t st) {
  return wkind == 0 ? launch_staged_nb<0>(P, mode, nb, cj, grid, st)
         : wkind == 1 ? launch_staged_nb<1>(P, mode, nb, cj, grid, st)
                      : launch_staged_nb<2>(P, mode, nb, cj, grid, st);
}

// Whole-row kernels (at most 16 tokens): rows of whole 256-byte multiples, for the compiled counts
// CH of 256-byte pieces per block column (bf16: K = 128 CH; 8-bit codes: K = 256 CH).
int rows4_chunks(int K, int wkind) {
  const int per = wkind ? 256 : 128;
  if (K % per != 0) return 0;
  const int ch = K / per;
  if (wkind) return (ch == 4 || ch == 5 || ch == 6 || ch == 8) ? ch : 0;
  return (ch == 4 || ch == 8 || ch == 10 || ch == 12 || ch == 16) ? ch : 0;
}
template <int WK, int NG, int CH, int NS>
hipError_t launch_rows4(const BatchParams& P, int mode, int tiles, hipStream_t st) {
  const size_t dyn = (size_t)CH * NG * (WK ? 2 : 1) * kWave * 16;
  const void* kern = mode == 0 ? reinterpret_cast<const void*>(predict_rows4_kernel<WK, NG, CH, NS>)
                               : reinterpret_cast<const void*>(k2_rows4_kernel<WK, NG, CH, NS>);
  const hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn);
  if (e != hipSuccess) return e;
  const dim3 grid((tiles + NS - 1) / NS, P.n_layers);
  if (mode == 0) hipLaunchKernelGGL((predict_rows4_kernel<WK, NG, CH, NS>), grid, dim3(kR4Threads), dyn, st, P);
  else hipLaunchKernelGGL((k2_rows4_kernel<WK, NG, CH, NS>), grid, dim3(kR4Threads), dyn, st, P);
  return hipGetLastError();
}
template <int WK, int NG, int CH>
hipError_t launch_rows4_ns(const BatchParams& P, int mode, bool brief, int tiles, hipStream_t st) {
  return brief ? launch_rows4<WK, NG, CH, 4>(P, mode, tiles, st) : launch_rows4<WK, NG, CH, 16>(P, mode, tiles, st);
}
template <int WK, int NG>
hipError_t launch_rows4_ch(const BatchParams& P, int mode, int ch, bool brief, int tiles, hipStream_t st) {
  if constexpr (WK == 0) {
    switch (ch) {
      case 4: return launch_rows4_ns<WK, NG, 4>(P, mode, brief, tiles, st);
      case 8: return launch_rows4_ns<WK, NG, 8>(P, mode, brief, tiles, st);
      case 10: return launch_rows4_ns<WK, NG, 10>(P, mode, brief, tiles, st);
      case 12: return launch_rows4_ns<WK, NG, 12>(P, mode, brief, tiles, st);
      case 16: return launch_rows4_ns<WK, NG, 16>(P, mode, brief, tiles, st);
      default: return hipErrorInvalidValue;
    }
  } else {
    switch (ch) {
      case 4: return launch_rows4_ns<WK, NG, 4>(P, mode, brief, tiles, st);
      case 5: return launch_rows4_ns<WK, NG, 5>(P, mode, brief, tiles, st);
      case 6: return launch_rows4_ns<WK, NG, 6>(P, mode, brief, tiles, st);
      case 8: return launch_rows4_ns<WK, NG, 8>(P, mode, brief, tiles, st);
      default: return hipErrorInvalidValue;
    }
  }
}
template <int WK>
hipError_t launch_rows4_ng(const BatchParams& P, int mode, int ch, bool brief, int tiles, hipStream_t st) {
  switch ((P.B + 3) / 4) {
    case 1: return launch_rows4_ch<WK, 1>(P, mode, ch, brief, tiles, st);
    case 2: return launch_rows4_ch<WK, 2>(P, mode, ch, brief, tiles, st);
    case 3: return launch_rows4_ch<WK, 3>(P, mode, ch, brief, tiles, st);
    case 4: return launch_rows4_ch<WK, 4>(P, mode, ch, brief, tiles, st);
    default: return hipErrorInvalidValue;
  }
}
hipError_t launch_rows4_wk(const BatchParams& P, int wkind, int mode, int ch, bool brief, int tiles, hipStream_t st) {
  return wkind == 0 ? launch_rows4_ng<0>(P, mode, ch, brief, tiles, st)
         : wkind == 1 ? launch_rows4_ng<1>(P, mode, ch, brief, tiles, st)
                      : launch_rows4_ng<2>(P, mode, ch, brief, tiles, st);
}

template <int NB, int WK>
hipError_t launch_v8(const BatchParams& P, dim3 grid, int nwv, size_t dyn, hipStream_t st) {
  const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(v_batch_kernel<NB, WK>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)((size_t)kVMaxWaves * 32 * kVPitch + (size_t)2 * planes_for(NB) * NB * kWave * 16));
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((v_batch_kernel<NB, WK>), grid, dim3(nwv * kWave), dyn, st, P);
  return hipGetLastError();
}

}  // namespace

size_t phased_batch_scratch_bytes(int d_model, int d_ff, int batch) { return batch_layout(d_model, d_ff, batch).total; }

bool phased_batch_supported(const FfnProblem& p) {
  const int r2 = p.d_model - p.r;
  int a = 0, b = 0;
  if (p.w_fp8) {
    // 8-bit codes: the whole-row kernels up to 16 tokens, the LDS-staged ones above (rows of whole 256-code multiples)
    const int nb = (p.batch + 15) / 16;
    const bool rows_ok = nb == 1 ? rows4_chunks(p.r, 1) > 0 && rows4_chunks(r2, 1) > 0 : staged_cj(p.r, nb) > 0 && staged_cj(r2, nb) > 0;
    return p.batch >= 2 && p.batch <= 64 && p.q_bf16 && rows_ok && p.d_model % 64 == 0 && p.d_ff <= 64 * kMaxWords && p.d_ff >= 16 &&
           (size_t)p.d_ff * (size_t)p.d_model < ((size_t)1 << 31);
  }
  return p.batch >= 2 && p.batch <= 64 && p.w_bf16 && p.q_bf16 && p.r % 32 == 0 && r2 % 32 == 0 &&
         p.d_model % 64 == 0 && p.d_ff <= 64 * kMaxWords && p.d_ff >= 16 && split_for(p.r, &a, &b) && split_for(r2, &a, &b) &&
         (size_t)p.d_ff * (size_t)p.d_model * 2 < ((size_t)1 << 31);  // 32-bit buffer offsets
}

hipError_t launch_ffn_phased_batch(const FfnProblem& p0, const void* const* k1n, const void* const* k2n,
                                   const void* const* vn, int n_layers, const FfnTuning& tune, void* scratch,
                                   hipStream_t st) {
  const BatchLayout lay = batch_layout(p0.d_model, p0.d_ff, p0.batch);
  // pinned choices (0 = automatic): tiles per workgroup of the predict and k2 steps (the block sizes
  // divided by 16); variant = 100 x kernel family + row slices of the V step.  Families: 0 automatic,
  // 1 the k-split kernels for every batch size, 4 the whole-row kernels wherever they are compiled,
  // 5 the LDS-staged kernels wherever they are compiled
  const int t1 = tune.rows_per_predict_block / 16, t2 = tune.neurons_per_gather_block / 16;
  const int family = tune.variant / 100;
  const int g_batch_ks = tune.variant % 100;
  const int g_batch_tpw1 = t1 > 0 ? (t1 + 3) / 4 * 4 : 0;
  const int g_batch_tpw2 = t2 > 0 ? min(32, (t2 + 3) / 4 * 4) : 0;
  char* s = static_cast<char*>(scratch);
  const int B = p0.batch, nb = (B + 15) / 16;
  hipError_t err = hipSuccess;
  // equal chunks of at most kBatchMaxLayers layers
  const int chunks = (n_layers + kBatchMaxLayers - 1) / kBatchMaxLayers, per = (n_layers + chunks - 1) / max(1, chunks);
  for (int base = 0; base < n_layers && err == hipSuccess; base += per) {
    const int L = min(per, n_layers - base);
    BatchParams P;
    for (int l = 0; l < kBatchMaxLayers; ++l) {
      P.k1n[l] = l < L ? k1n[base + l] : nullptr;
      P.k2n[l] = l < L ? k2n[base + l] : nullptr;
      P.vn[l] = l < L ? vn[base + l] : nullptr;
    }
    P.q = static_cast<const bf16_t*>(p0.q) + (size_t)base * p0.q_slot_stride;
    P.qslot = p0.q_slot_stride;
    P.ldq = p0.ldq;
    P.y = p0.y + (size_t)base * B * p0.d_model;
    P.theta = p0.theta ? p0.theta + (size_t)base * B : nullptr;
    P.count = p0.active_count ? p0.active_count + (size_t)base * B : nullptr;
    P.idx = p0.active_idx ? p0.active_idx + (size_t)base * B * p0.d_ff : nullptr;
    P.ucount = p0.union_count ? p0.union_count + base : nullptr;
    P.uidx = p0.union_idx ? p0.union_idx + (size_t)base * p0.d_ff : nullptr;
    P.S = reinterpret_cast<float*>(s + lay.S);
    P.ST = reinterpret_cast<float*>(s + lay.ST);
    P.BP = (B + 15) / 16 * 16;
    P.thetas = reinterpret_cast<float*>(s + lay.thetas);
    P.tmask = reinterpret_cast<unsigned long long*>(s + lay.tmask);
    P.urow = reinterpret_cast<int32_t*>(s + lay.urow);
    P.utotal = reinterpret_cast<int32_t*>(s + lay.utotal);
    P.up = reinterpret_cast<uint16_t*>(s + lay.up);
    P.plane = lay.plane;
    P.part = reinterpret_cast<float*>(s + lay.part);
    P.n_layers = L;
    P.B = B;
    P.d_model = p0.d_model;
    P.d_ff = p0.d_ff;
    P.r = p0.r;
    P.gelu = p0.gelu;
    P.ldu = lay.ldu;
    P.planes = planes_for(nb);
    P.z = p0.z;
    const int tiles = (p0.d_ff + 15) / 16;
    int tpw1 = 16;  // multiples of 4 (the deepest tile pipeline)
    while (tpw1 > 4 && (long long)L * ((tiles + tpw1 - 1) / tpw1) < 768) tpw1 /= 2;
    int tpw2 = 16;  // long ranges amortise the rank lookup of a k2 workgroup
    while (tpw2 > 4 && (long long)L * ((tiles + tpw2 - 1) / tpw2) < 512) tpw2 /= 2;
    if (g_batch_tpw1 > 0) tpw1 = g_batch_tpw1;
    if (g_batch_tpw2 > 0) tpw2 = g_batch_tpw2;
    P.TPW1 = tpw1;
    P.TPW2 = tpw2;
    const int slabs = v_slabs(p0.d_model, nb);
    // Row slices: a workgroup's time is its share of the rows plus a fixed part (start-up and
    // its partial sums, about 2 % of a whole column slab), and the launch takes as many rounds
    // as its workgroups need of the chip's resident slots; take the cheapest count.
    const int v_slots = 256 * max(1, 4 * (nb == 4 ? 2 : nb == 3 ? 3 : 4) / v_waves(p0.d_model, nb));
    int ksl = 1;
    double cost_best = 1e30;
    for (int c = 1; c <= 16 && L * c <= part_rows(p0.d_model); ++c) {
      const long long n = (long long)slabs * L * c;
      const double cost = (double)((n + v_slots - 1) / v_slots) * (1.0 / c + 0.02);
      if (cost < cost_best) { cost_best = cost; ksl = c; }
    }
    if (g_batch_ks > 0) ksl = g_batch_ks;
    ksl = max(1, min(16, ksl));
    while (L * ksl > part_rows(p0.d_model)) --ksl;
    P.KS = ksl;

    // Which predict / k2 kernels: the whole-row kernels with at most 16 tokens and rows of whole
    // 256-byte multiples, as long as the tokens' operands (a KB per 128 elements of a row and group
    // of four tokens) leave room for three workgroups per compute unit; the LDS-staged kernels with
    // more tokens, or where the whole-row ones do not fit, for rows of whole 512-byte multiples; the
    // k-split kernels for everything else.  A pair that both read the token-major scores leaves the
    // neuron-major copy unwritten.  8-bit codes exist for the first two families only.
    const bool few_wgs = (long long)L * ((tiles + 15) / 16) < 600;
    const int wkind = p0.w_fp8;  // 0 bf16, 1 E4M3 codes, 2 integer codes
    const int ngrp = (B + 3) / 4;
    const bool pieces_only = family == 1 && !wkind;
    int ch1 = nb == 1 && !pieces_only && family != 5 ? rows4_chunks(p0.r, wkind) : 0;
    int ch2 = nb == 1 && !pieces_only && family != 5 ? rows4_chunks(p0.d_model - p0.r, wkind) : 0;
    if (family != 4 && !wkind) {
      if (ch2 * ngrp > 40) ch2 = 0;
      if (ch1 * ngrp > 48) ch1 = 0;
    }
    if (ch1 == 0 || ch2 == 0) ch1 = ch2 = 0;  // (the two steps change over together)
    const bool staged_on = !pieces_only && ch1 == 0;
    const int cj1 = staged_on ? staged_cj(p0.r, nb) : 0, cj2 = staged_on ? staged_cj(p0.d_model - p0.r, nb) : 0;
    if (wkind && ch1 == 0 && (cj1 == 0 || cj2 == 0)) return hipErrorInvalidValue;
    // workgroups of 64 rows up to 8 tokens, of 256 above (measured on the 2B, 9B and paper shapes)
    const bool r4_short1 = g_batch_tpw1 > 0 ? g_batch_tpw1 < 16 : (few_wgs || ngrp <= 2);
    const bool r4_short2 = g_batch_tpw2 > 0 ? g_batch_tpw2 < 16 : (few_wgs || ngrp <= 2);
    if (ch1 > 0) {
      BatchParams P1 = P;
      P1.ST = nullptr;
      err = launch_rows4_wk(P1, wkind, 0, ch1, r4_short1, tiles, st);
    } else if (cj1 > 0) {
      BatchParams P1 = P;
      if (cj2 > 0) P1.ST = nullptr;
      err = launch_staged_wk(P1, wkind, 0, nb, cj1, dim3((tiles + tpw1 - 1) / tpw1, L), st);
    } else {
      err = launch_rows_nb(P, 0, nb, p0.r, dim3((tiles + tpw1 - 1) / tpw1, L), st);
    }
    if (err != hipSuccess) return err;
    if (p0.d_ff <= 36 * kSelThreads) hipLaunchKernelGGL((select_batch_kernel<36>), dim3(B, L), dim3(kSelThreads), 0, st, P);
    else hipLaunchKernelGGL((select_batch_kernel<64>), dim3(B, L), dim3(kSelThreads), 0, st, P);
    hipLaunchKernelGGL(union_batch_kernel, dim3(L), dim3(4 * kMaxWords), 0, st, P);
    if (ch2 > 0) {
      P.TPW2 = r4_short2 ? 4 : 16;
      err = launch_rows4_wk(P, wkind, 1, ch2, r4_short2, tiles, st);
    } else if (cj2 > 0) {
      err = launch_staged_wk(P, wkind, 1, nb, cj2, dim3((tiles + tpw2 - 1) / tpw2, L), st);
    } else {
      err = launch_rows_nb(P, 1, nb, p0.d_model - p0.r, dim3((tiles + tpw2 - 1) / tpw2, L), st);
    }
    if (err != hipSuccess) return err;
    P.VSLABS = slabs;
    const dim3 gv((unsigned)(((long long)slabs * ksl * L + 7) / 8 * 8));  // (a whole number of rounds over the dies)
    const int nwv = v_waves(p0.d_model, nb);
    const size_t vdyn = (size_t)nwv * 32 * kVPitch + (size_t)2 * planes_for(nb) * nb * kWave * 16;
    const void* vk = nb == 1 ? reinterpret_cast<const void*>(v_batch_kernel<1>)
                     : nb == 2 ? reinterpret_cast<const void*>(v_batch_kernel<2>)
                     : nb == 3 ? reinterpret_cast<const void*>(v_batch_kernel<3>)
                               : reinterpret_cast<const void*>(v_batch_kernel<4>);
    // (the attribute is set to the most this variant can ask for, the same value on every call)
    err = hipFuncSetAttribute(vk, hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)((size_t)kVMaxWaves * 32 * kVPitch + (size_t)2 * planes_for(nb) * nb * kWave * 16));
    if (err != hipSuccess) return err;
    if (wkind) {
      err = wkind == 1 ? (nb == 1 ? launch_v8<1, 1>(P, gv, nwv, vdyn, st) : nb == 2 ? launch_v8<2, 1>(P, gv, nwv, vdyn, st)
                          : nb == 3 ? launch_v8<3, 1>(P, gv, nwv, vdyn, st) : launch_v8<4, 1>(P, gv, nwv, vdyn, st))
                       : (nb == 1 ? launch_v8<1, 2>(P, gv, nwv, vdyn, st) : nb == 2 ? launch_v8<2, 2>(P, gv, nwv, vdyn, st)
                          : nb == 3 ? launch_v8<3, 2>(P, gv, nwv, vdyn, st) : launch_v8<4, 2>(P, gv, nwv, vdyn, st));
      if (err != hipSuccess) return err;
    } else
    switch (nb) {
      case 1: hipLaunchKernelGGL((v_batch_kernel<1>), gv, dim3(nwv * kWave), vdyn, st, P); break;
      case 2: hipLaunchKernelGGL((v_batch_kernel<2>), gv, dim3(nwv * kWave), vdyn, st, P); break;
      case 3: hipLaunchKernelGGL((v_batch_kernel<3>), gv, dim3(nwv * kWave), vdyn, st, P); break;
      default: hipLaunchKernelGGL((v_batch_kernel<4>), gv, dim3(nwv * kWave), vdyn, st, P); break;
    }
    const size_t n = (size_t)B * p0.d_model;
    hipLaunchKernelGGL(reduce_batch_kernel, dim3((unsigned)((n + 255) / 256), L), dim3(256), 0, st, P);
    err = hipGetLastError();
  }
  return err;
}

}  // namespace spark
