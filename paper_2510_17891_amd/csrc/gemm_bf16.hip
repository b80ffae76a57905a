// Weight-streaming bf16 GEMM for decode-sized batches:  Y[M x N] = X[M x K] * W[N x K]^T.
//
// At M <= 256 the projection is bound by reading W once from HBM (M flop per weight byte), so the kernel is
// organised around that stream: both operands are stored fragment-major (see frag_offset), which makes every
// global load a fully coalesced 1 KiB wave access that lands directly in MFMA 32x32x16 operand registers (the packed
// weights hold the f16 image of the model's bf16 weights; the activations arrive as f16) -- no LDS staging, no shuffles.  A wave owns a 64 x (32*MB) output tile over a slice of K; the four waves of a
// block take four K slices and add their accumulators through LDS in a fixed order; further K splits across
// blocks (to put >= 256 blocks on the chip for the small matrices) leave fp32 partials that the consumer sums.
#include <type_traits>

#include "device_utils.h"
#include "kernels.h"
#include "sampler_device.h"

namespace rl {

namespace {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ f32x16_t mfma_f16(u32x4_t a, u32x4_t b, f32x16_t c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
}

template <int MB, int RB = 2>
struct Frags {
  u32x4_t a[RB][4];  // RB 32-row blocks of the weight matrix
  u32x4_t b[MB][4];
};

// wr[nb]: row block nb of the tile; NT: weights pass through once (non-temporal), otherwise the block's other waves
// read the same tile and it may live in L1/L2.
// kb: the k block (activations are stored in that order); kw: where the weights keep it (weight_kb_slot).
template <int MB, int RB, bool NT = true>
__device__ __forceinline__ void load_frags(Frags<MB, RB>& f, const u32x4_t* const (&wr)[RB],
                                           const u32x4_t* const* __restrict__ xb, int kb, int kw, int lane) {
  // block (rb, slot) = 256 uint4; sub-load t is [t*64 + lane]
  const int o = kb * 256 + lane, ow = kw * 256 + lane;
#pragma unroll
  for (int t = 0; t < 4; ++t) {
#pragma unroll
    for (int nb = 0; nb < RB; ++nb) f.a[nb][t] = NT ? __builtin_nontemporal_load(wr[nb] + ow + t * 64) : wr[nb][ow + t * 64];
  }
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int t = 0; t < 4; ++t) f.b[mb][t] = xb[mb][o + t * 64];
}

template <int MB, int RB>
__device__ __forceinline__ void mma_frags(const Frags<MB, RB>& f, f32x16_t (&acc)[RB][MB]) {
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int nb = 0; nb < RB; ++nb) {
      const u32x4_t a = f.a[nb][t];
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) acc[nb][mb] = mfma_f16(a, f.b[mb][t], acc[nb][mb]);
    }
}

// One finished 32-row block held in MFMA accumulator order -- lane (col, hb) has outputs 8q + 4hb + e (q, e = 0..3)
// of batch row m -- for the epilogues that work per row block.
template <int EPI>
__device__ __forceinline__ void store_rowblock(const float (&sum)[16], int m, int hb, int rb, int split, int M, int N,
                                               void* __restrict__ out) {
  if (EPI == kEpiPartial) {
    float* o = (float*)out + ((size_t)split * M + m) * N;
#pragma unroll
    for (int q = 0; q < 4; ++q)
      *(float4*)(o + rb * 32 + 8 * q + 4 * hb) = make_float4(sum[4 * q], sum[4 * q + 1], sum[4 * q + 2], sum[4 * q + 3]);
  } else {
    // SwiGLU: a 32-row block of the interleaved gate/up matrix holds the gate rows (0..15) and the up rows (16..31)
    // of the 16 outputs 16 rb .. 16 rb + 15: a lane finds both factors of its outputs in its own registers.
    uint16_t* o = (uint16_t*)out;
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      float a[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float gte = sum[4 * q + e], up = sum[4 * (q + 2) + e];
        a[e] = gte / (1.0f + __expf(-gte)) * up;
      }
      *(uint2*)(o + frag_offset(m, rb * 16 + 8 * q + 4 * hb, N >> 6)) = make_uint2(pack2h(a[0], a[1]), pack2h(a[2], a[3]));
    }
  }
}

// Write one finished 64 x 32 output block held in MFMA accumulator order: lane (col, hb) has, for both row blocks,
// outputs n = rb*32 + 8q + 4hb + e (q, e = 0..3) of batch row m.
template <int EPI>
__device__ __forceinline__ void store_block(const float (&sum)[2][16], int m, int hb, int rb0, int rb1, int split, int M,
                                          int N, void* __restrict__ out, const SampleEpilogue& se, int tile) {
  if (EPI == kEpiPartial || EPI == kEpiSwiGLU) {
    store_rowblock<EPI>(sum[0], m, hb, rb0, split, M, N, out);
    store_rowblock<EPI>(sum[1], m, hb, rb1, split, M, N, out);
  } else {
    // lane (col, hb) holds 32 logits of row m: vocabulary ids (rb*32 + 8q + 4hb + e), in aligned groups of four,
    // i.e. one Philox block per group.
    const RowMeta rm = se.rows[m];
    const uint32_t pos = (uint32_t)(rm.pos + se.pos_offset), seq = (uint32_t)rm.seq;
    const int f = se.forced ? se.forced[m] : -1;
    Best best{-INFINITY, -1, 0.f};
    // log-sum-exp of the lane's 32 entries: their maximum first, then one exponential per entry
    float lm = -INFINITY, ls = 0.f;
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int r = 0; r < 16; ++r) lm = fmaxf(lm, sum[nb][r] * se.inv_t);
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n0 = (nb ? rb1 : rb0) * 32 + 8 * q + 4 * hb;
        uint32_t rnd[4] = {0, 0, 0, 0};
        if (!se.greedy) philox4x32_10((uint32_t)n0 >> 2, pos, seq, 0u, se.seed_lo, se.seed_hi, rnd);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float zi = sum[nb][4 * q + e];
          const float y = se.greedy ? zi : __fmaf_rn(zi, se.inv_t, gumbel(rnd[e]));
          best = better(best, Best{y, n0 + e, zi});
          if (lm != -INFINITY) ls += __expf(zi * se.inv_t - lm);
          if (n0 + e == f) se.forced_z[m] = zi;
        }
        if (se.logits_out)
          *(float4*)(se.logits_out + (size_t)m * N + n0) =
              make_float4(sum[nb][4 * q], sum[nb][4 * q + 1], sum[nb][4 * q + 2], sum[nb][4 * q + 3]);
      }
    best = better(best, shfl_xor_best(best, 32));  // the other half of this row's 64 entries
    lse_merge(lm, ls, __shfl_xor(lm, 32, kWave), __shfl_xor(ls, 32, kWave));
    if (hb == 0) {
      float* p = se.part + ((size_t)m * (N >> 6) + tile) * kSamplePartFloats;
      *(float4*)p = make_float4(best.y, __int_as_float(best.idx), best.z, 0.f);
      *(float4*)(p + 4) = make_float4(lm, ls, 0.f, 0.f);
    }
  }
}

// grid: x = N tile, y = K split, z = M tile of 32*MB rows.
//   EPI == kEpiPartial: tile = 64 output columns (row blocks 2x, 2x+1 of W); out fp32 [S][M][N].
//   EPI == kEpiSwiGLU : tile = 32 output columns (row blocks 2x, 2x+1 of the interleaved gate/up matrix, each 16 gate
//                       rows and the 16 up rows of the same outputs); out f16 fragment-major [M x N].
//   EPI == kEpiSample : tile = 64 vocabulary entries; the logits stay in registers: temperature, Gumbel noise, running
//                       arg-max and log-sum-exp are taken per (row, tile) and only those partials are written
//                       (plus the logits themselves when the caller asked for them).
// ST = k blocks a wave keeps in flight.  HBM latency is ~10x the MFMA time of a block, so the loop is a ring of
// ST register buffers: compute block i, immediately re-issue its buffer for block i + ST.  The scheduling
// barriers keep the compiler from sinking the loads below the next block's MFMAs.
// One tile of RB 32-row blocks (rb_first .. rb_first + RB - 1) over the K range of `split`, for batch tile m_tile:
// the body of the K-split kernels.  `tile` is the index of the 64-entry vocabulary tile (sampling epilogue, RB == 2).
template <int MB, int EPI, int ST, int RB>
__device__ __forceinline__ void kslice_tile(const u32x4_t* __restrict__ X, const u32x4_t* __restrict__ W,
                                            void* __restrict__ out, int M, int N, int K, int kb_per_wave,
                                            const SampleEpilogue& se, int rb_first, int split, int m_tile, int tile,
                                            float (&red)[4][16][64]) {
  static_assert(EPI != kEpiSample || RB == 2, "the sampling epilogue works on 64-entry tiles");
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int KB = K >> 6;
  const int m_blk0 = m_tile * MB;
  const int n_blocks_m = (M + 31) >> 5;
  const u32x4_t* wr[RB];
#pragma unroll
  for (int nb = 0; nb < RB; ++nb) wr[nb] = W + (size_t)(rb_first + nb) * KB * 256;
  const u32x4_t* xb[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    int b = m_blk0 + mb;
    if (b >= n_blocks_m) b = n_blocks_m - 1;  // clamp: surplus column blocks are computed but never stored
    xb[mb] = X + (size_t)b * KB * 256;
  }

  f32x16_t acc[RB][MB];
#pragma unroll
  for (int nb = 0; nb < RB; ++nb)
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[nb][mb][r] = 0.f;

  const int kb0 = (split * 4 + wave) * kb_per_wave;
  const int kw0 = split * 4 * kb_per_wave + wave;  // slot of k block kb0; this wave's later blocks follow at stride 4
  const int n = kb_per_wave;
  Frags<MB, RB> f[ST];
#pragma unroll
  for (int s = 0; s < ST; ++s) load_frags<MB, RB>(f[s], wr, xb, kb0 + s, kw0 + 4 * s, lane);  // the launcher guarantees ST <= n
  const int full = n / ST, rem = n - full * ST;
  int b = 0;
  for (int r = 0; r + 1 < full; ++r) {  // steady state: every buffer is refilled
#pragma unroll
    for (int s = 0; s < ST; ++s) {
      mma_frags<MB, RB>(f[s], acc);
      __builtin_amdgcn_sched_barrier(0);
      load_frags<MB, RB>(f[s], wr, xb, kb0 + b + s + ST, kw0 + 4 * (b + s + ST), lane);
      __builtin_amdgcn_sched_barrier(0);
    }
    b += ST;
  }
  if (full > 0) {  // last full round: refill only what the remainder round will use
#pragma unroll
    for (int s = 0; s < ST; ++s) {
      mma_frags<MB, RB>(f[s], acc);
      __builtin_amdgcn_sched_barrier(0);
      if (s < rem) load_frags<MB, RB>(f[s], wr, xb, kb0 + b + s + ST, kw0 + 4 * (b + s + ST), lane);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
#pragma unroll
  for (int s = 0; s < ST; ++s)
    if (s < rem) mma_frags<MB, RB>(f[s], acc);

  // ---- add the four waves' accumulators (fixed order) and write: column block mb is finished by wave mb % 4 ----
  const int col = lane & 31, hb = lane >> 5;
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    float sum[RB][16];
#pragma unroll
    for (int nb = 0; nb < RB; ++nb) {
      __syncthreads();
#pragma unroll
      for (int r = 0; r < 16; ++r) red[wave][r][lane] = acc[nb][mb][r];
      __syncthreads();
      if (wave == (mb & 3)) {
#pragma unroll
        for (int r = 0; r < 16; ++r)
          sum[nb][r] = ((red[0][r][lane] + red[1][r][lane]) + red[2][r][lane]) + red[3][r][lane];
      }
    }
    if (wave != (mb & 3)) continue;
    const int m = (m_blk0 + mb) * 32 + col;
    if (m >= M) continue;
    if constexpr (EPI == kEpiSample) {
      store_block<EPI>(sum, m, hb, rb_first, rb_first + 1, split, M, N, out, se, tile);
    } else {
#pragma unroll
      for (int nb = 0; nb < RB; ++nb) store_rowblock<EPI>(sum[nb], m, hb, rb_first + nb, split, M, N, out);
    }
  }
}

template <int MB, int EPI, int ST>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(const u32x4_t* __restrict__ X, const u32x4_t* __restrict__ W,
                                                        void* __restrict__ out, int M, int N, int K, int kb_per_wave,
                                                        SampleEpilogue se) {
  __shared__ float red[4][16][64];
  kslice_tile<MB, EPI, ST, 2>(X, W, out, M, N, K, kb_per_wave, se, blockIdx.x * 2, blockIdx.y, blockIdx.z, blockIdx.x, red);
}

// The same with tiles of two sizes in one launch, for matrices whose row blocks times K splits are three per compute
// unit (768 on this chip): n_big tiles of two row blocks per split come first in the grid, then n_small tiles of one.
// Two blocks fit a compute unit, and blocks are handed out in grid order to whatever unit has room: the first 256 land
// one per unit, the second 256 fill the remaining place of each, so every unit streams three row blocks -- the same
// bytes everywhere -- with two blocks resident, each hiding the other's start and end.  (Tiles of one size leave either
// 384 blocks, i.e. half of the units with twice the bytes of the rest, or 256 with nothing to overlap.)  Same K
// ranges, same order: same bits as every other variant.
// grid: x = splits * (n_big + n_small), z = M tile of 32*MB rows.
template <int MB, int EPI, int ST>
__global__ __launch_bounds__(256) void gemm_bf16_mixed_kernel(const u32x4_t* __restrict__ X, const u32x4_t* __restrict__ W,
                                                              void* __restrict__ out, int M, int N, int K, int kb_per_wave,
                                                              int n_big, int n_small, int splits, SampleEpilogue se) {
  static_assert(EPI != kEpiSample, "per-row-block epilogues only");
  __shared__ float red[4][16][64];
  const int id = blockIdx.x, all_big = splits * n_big;  // block-uniform
  if (id < all_big) {
    kslice_tile<MB, EPI, ST, 2>(X, W, out, M, N, K, kb_per_wave, se, (id % n_big) * 2, id / n_big, blockIdx.z, 0, red);
  } else {
    const int j = id - all_big;
    kslice_tile<MB, EPI, ST, 1>(X, W, out, M, N, K, kb_per_wave, se, 2 * n_big + j % n_small, j / n_small, blockIdx.z, 0, red);
  }
}

// The K-split kernel with a 128-row weight tile (two 64-row pairs, four 32-row blocks per wave).  Every block reads
// the whole activation panel once, so halving the number of blocks halves that traffic; from about 48 rows on the
// panel reads of the 64-row tiling are as large as the weight stream itself and the launch is bound by what L2
// delivers.  Used where the halved grid still fills the chip.  Same K ranges per wave, same order: same bits.
template <int MB>
struct FragsW {
  u32x4_t a[4][4];
  u32x4_t b[MB][4];
};

template <int MB, int EPI, int ST>
__global__ __launch_bounds__(256, 1) void gemm_bf16_wide_kernel(const u32x4_t* __restrict__ X, const u32x4_t* __restrict__ W,
                                                              void* __restrict__ out, int M, int N, int K, int kb_per_wave,
                                                              SampleEpilogue se) {
  __shared__ float red[4][16][64];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int KB = K >> 6;
  const int m_blk0 = blockIdx.z * MB;
  const int n_blocks_m = (M + 31) >> 5;
  const int n_tiles = EPI == kEpiSwiGLU ? (N >> 5) : (N >> 6);
  int tile[2], rb[4];
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    tile[p] = min((int)blockIdx.x * 2 + p, n_tiles - 1);  // an odd tile count: the last block's second pair shadows its first
    rb[2 * p] = tile[p] * 2;
    rb[2 * p + 1] = tile[p] * 2 + 1;
  }
  const bool second_valid = (int)blockIdx.x * 2 + 1 < n_tiles;
  const u32x4_t* wp[4];
#pragma unroll
  for (int b = 0; b < 4; ++b) wp[b] = W + (size_t)rb[b] * KB * 256 + lane;
  const u32x4_t* xb[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    int b = m_blk0 + mb;
    if (b >= n_blocks_m) b = n_blocks_m - 1;  // clamp: surplus column blocks are computed but never stored
    xb[mb] = X + (size_t)b * KB * 256 + lane;
  }
  f32x16_t acc[4][MB];
#pragma unroll
  for (int b = 0; b < 4; ++b)
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[b][mb][r] = 0.f;

  const int kw0 = blockIdx.y * 4 * kb_per_wave + wave - 4 * ((blockIdx.y * 4 + wave) * kb_per_wave);  // slot = kw0 + 4 kb
  auto load = [&](FragsW<MB>& f, int kb) __attribute__((always_inline)) {
    const int o = kb * 256, ow = (kw0 + 4 * kb) * 256;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
#pragma unroll
      for (int b = 0; b < 4; ++b) f.a[b][t] = __builtin_nontemporal_load(wp[b] + ow + t * 64);
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) f.b[mb][t] = xb[mb][o + t * 64];
    }
  };
  auto mma = [&](const FragsW<MB>& f) __attribute__((always_inline)) {
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const u32x4_t a = f.a[b][t];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) acc[b][mb] = mfma_f16(a, f.b[mb][t], acc[b][mb]);
      }
  };

  const int kb0 = (blockIdx.y * 4 + wave) * kb_per_wave;
  const int n = kb_per_wave;
  FragsW<MB> f[ST];
#pragma unroll
  for (int s = 0; s < ST; ++s) load(f[s], kb0 + s);  // the launcher guarantees ST <= n
  const int full = n / ST, rem = n - full * ST;
  int b = 0;
  for (int r = 0; r + 1 < full; ++r) {  // steady state: every buffer is refilled
#pragma unroll
    for (int s = 0; s < ST; ++s) {
      mma(f[s]);
      __builtin_amdgcn_sched_barrier(0);
      load(f[s], kb0 + b + s + ST);
      __builtin_amdgcn_sched_barrier(0);
    }
    b += ST;
  }
  if (full > 0) {  // last full round: refill only what the remainder round will use
#pragma unroll
    for (int s = 0; s < ST; ++s) {
      mma(f[s]);
      __builtin_amdgcn_sched_barrier(0);
      if (s < rem) load(f[s], kb0 + b + s + ST);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
#pragma unroll
  for (int s = 0; s < ST; ++s)
    if (s < rem) mma(f[s]);

  // ---- add the four waves' accumulators (fixed order) and write: column block mb is finished by wave mb % 4 ----
  const int col = lane & 31, hb = lane >> 5;
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    float sum[4][16];
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) {
      __syncthreads();
#pragma unroll
      for (int r = 0; r < 16; ++r) red[wave][r][lane] = acc[nb][mb][r];
      __syncthreads();
      if (wave == (mb & 3)) {
#pragma unroll
        for (int r = 0; r < 16; ++r)
          sum[nb][r] = ((red[0][r][lane] + red[1][r][lane]) + red[2][r][lane]) + red[3][r][lane];
      }
    }
    if (wave != (mb & 3)) continue;
    const int m = (m_blk0 + mb) * 32 + col;
    if (m >= M) continue;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      if (p == 1 && !second_valid) break;
      float pair[2][16];
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r) pair[nb][r] = sum[2 * p + nb][r];
      store_block<EPI>(pair, m, hb, rb[2 * p], rb[2 * p + 1], blockIdx.y, M, N, out, se, tile[p]);
    }
  }
}

// Variant for 64 < M <= 256: the four waves take different batch-column blocks (MBW blocks of 32 each) instead of
// different K quarters, so a wave needs only 32*MBW accumulator columns and the block still streams W once (the
// four waves read the same weight tile at about the same time; only the first read leaves L2).  To keep a row's
// result bit-identical to the K-split variants, every wave still forms the four K-quarter sums separately and adds
// them in that order, ((q0 + q1) + q2) + q3, which needs two accumulator sets.
template <int MBW, int EPI, int ST>
__global__ __launch_bounds__(256) void gemm_bf16_cols_kernel(const u32x4_t* __restrict__ X, const u32x4_t* __restrict__ W,
                                                             void* __restrict__ out, int M, int N, int K, int kb_per_quarter,
                                                             SampleEpilogue se) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int KB = K >> 6;
  const int m_blk0 = (blockIdx.z * 4 + wave) * MBW;
  const int n_blocks_m = (M + 31) >> 5;
  if (m_blk0 >= n_blocks_m) return;  // this wave has no rows (no barriers below)

  int rb0, rb1;
  rb0 = blockIdx.x * 2;  // SwiGLU: the gate/up matrix is interleaved in 16-row groups, so this holds for it too
  rb1 = rb0 + 1;
  const u32x4_t* const wr[2] = {W + (size_t)rb0 * KB * 256, W + (size_t)rb1 * KB * 256};
  const u32x4_t* xb[MBW];
#pragma unroll
  for (int mb = 0; mb < MBW; ++mb) {
    int b = m_blk0 + mb;
    if (b >= n_blocks_m) b = n_blocks_m - 1;
    xb[mb] = X + (size_t)b * KB * 256;
  }
  const int kb0 = blockIdx.y * 4 * kb_per_quarter;
  const int rounds = kb_per_quarter / ST;  // the launcher picks ST so that it divides kb_per_quarter
  Frags<MBW> f[ST];
  auto slot = [&](int kb) { return weight_kb_slot(kb, kb_per_quarter); };
#pragma unroll
  for (int s = 0; s < ST; ++s) load_frags<MBW, 2, false>(f[s], wr, xb, kb0 + s, slot(kb0 + s), lane);
  // One K quarter into a fresh accumulator.  The register ring keeps running across quarters: every block but the
  // last ST of the whole range re-issues its buffer for the block ST ahead.
  auto quarter = [&](f32x16_t (&a)[2][MBW], int q, bool last) __attribute__((always_inline)) {
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int mb = 0; mb < MBW; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) a[nb][mb][r] = 0.f;
    const int base = kb0 + q * kb_per_quarter;
    const int refill_rounds = last ? rounds - 1 : rounds;
    for (int r = 0; r < refill_rounds; ++r) {
#pragma unroll
      for (int s = 0; s < ST; ++s) {
        mma_frags<MBW, 2>(f[s], a);
        __builtin_amdgcn_sched_barrier(0);
        load_frags<MBW, 2, false>(f[s], wr, xb, base + r * ST + s + ST, slot(base + r * ST + s + ST), lane);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    if (last) {
#pragma unroll
      for (int s = 0; s < ST; ++s) mma_frags<MBW, 2>(f[s], a);
    }
  };
  f32x16_t acc[2][MBW], other[2][MBW];
  quarter(acc, 0, false);
#pragma unroll
  for (int q = 1; q < 4; ++q) {
    quarter(other, q, q == 3);
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int mb = 0; mb < MBW; ++mb) acc[nb][mb] += other[nb][mb];
  }

  const int col = lane & 31, hb = lane >> 5;
#pragma unroll
  for (int mb = 0; mb < MBW; ++mb) {
    const int m = (m_blk0 + mb) * 32 + col;
    if (m >= M) continue;
    float sum[2][16];
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int r = 0; r < 16; ++r) sum[nb][r] = acc[nb][mb][r];
    store_block<EPI>(sum, m, hb, rb0, rb1, blockIdx.y, M, N, out, se, blockIdx.x);
  }
}

// Variant of the column-split kernel that fetches every weight tile from global memory once per block: the 256
// threads copy the tile (two 32-row blocks x 64 k = 8 KiB) into one of four LDS stages, one barrier per k block
// publishes it, and each wave reads its MFMA A fragments from LDS while its own activation fragments keep coming
// straight from L2.  Weight registers run four k blocks ahead of the LDS stage they feed.  Needs K quarters that
// are multiples of four k blocks (true for every 8B-shaped matrix); same quarter arithmetic, same bits.
template <int MBW, int EPI, int XS>
__global__ __launch_bounds__(256, MBW == 1 ? 2 : 1) void gemm_bf16_lds_kernel(const u32x4_t* __restrict__ X,
                                                                           const u32x4_t* __restrict__ W,
                                                                           void* __restrict__ out, int M, int N, int K,
                                                                           int kb_per_quarter, SampleEpilogue se) {
  __shared__ u32x4_t wlds[4][2][256];  // 32 KiB
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int KB = K >> 6;
  const int n_blocks_m = (M + 31) >> 5;
  int m_blk0 = (blockIdx.z * 4 + wave) * MBW;
  const bool has_rows = m_blk0 < n_blocks_m;
  if (!has_rows) m_blk0 = n_blocks_m - 1;  // idle waves shadow a valid block (they still carry tiles and barriers)

  int rb0, rb1;
  rb0 = blockIdx.x * 2;  // SwiGLU: the gate/up matrix is interleaved in 16-row groups, so this holds for it too
  rb1 = rb0 + 1;
  const u32x4_t* w0 = W + (size_t)rb0 * KB * 256 + tid;
  const u32x4_t* w1 = W + (size_t)rb1 * KB * 256 + tid;
  const u32x4_t* xb[MBW];
#pragma unroll
  for (int mb = 0; mb < MBW; ++mb) {
    int b = m_blk0 + mb;
    if (b >= n_blocks_m) b = n_blocks_m - 1;
    xb[mb] = X + (size_t)b * KB * 256 + lane;
  }
  const int n = 4 * kb_per_quarter;
  const int kb0 = blockIdx.y * n;
  auto kb_of = [&](int i) { return kb0 + (i < n ? i : n - 1); };  // clamped: no conditional loads in the pipeline
  // Weight k blocks are loaded strictly in order (0, 1, 2, ...; the last one again once the range is exhausted), so
  // the slot of the next one is kept as (block within its quarter, quarter) and stepped, without a division.
  int w_r = 0, w_q = 0;
  auto next_wslot = [&]() {
    const int off = (((int)blockIdx.y * kb_per_quarter + w_r) * 4 + w_q) * 256;
    if (w_r + 1 < kb_per_quarter) ++w_r;
    else if (w_q < 3) { w_r = 0; ++w_q; }
    return off;
  };

  u32x4_t wr[4][2];          // weight registers: slot s holds a block with index = s (mod 4)
  u32x4_t xr[XS][MBW][4];    // activation fragments: slot s holds a block with index = s (mod XS)
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const int ow = next_wslot();
    wr[s][0] = __builtin_nontemporal_load(w0 + ow);
    wr[s][1] = __builtin_nontemporal_load(w1 + ow);
  }
#pragma unroll
  for (int s = 0; s < XS; ++s)
#pragma unroll
    for (int mb = 0; mb < MBW; ++mb)
#pragma unroll
      for (int t = 0; t < 4; ++t) xr[s][mb][t] = xb[mb][(size_t)kb_of(s) * 256 + t * 64];
  wlds[0][0][tid] = wr[0][0];
  wlds[0][1][tid] = wr[0][1];
  {
    const int ow = next_wslot();
    wr[0][0] = __builtin_nontemporal_load(w0 + ow);
    wr[0][1] = __builtin_nontemporal_load(w1 + ow);
  }

  // One k block: publish the next tile, barrier, multiply this one.  j = i mod 4 at compile time.
  auto iter = [&](f32x16_t (&a)[2][MBW], int i, auto jc) __attribute__((always_inline)) {
    constexpr int j = decltype(jc)::value, jn = (j + 1) & 3, jx = j % XS;
    wlds[jn][0][tid] = wr[jn][0];
    wlds[jn][1][tid] = wr[jn][1];
    const int ow = next_wslot();  // k block i + 5
    wr[jn][0] = __builtin_nontemporal_load(w0 + ow);
    wr[jn][1] = __builtin_nontemporal_load(w1 + ow);
    // Barrier that orders LDS traffic only: __syncthreads() would also drain every global load in flight
    // (loads and stores share one counter on this ISA), i.e. the whole prefetch pipeline, once per k block.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const u32x4_t a0 = wlds[j][0][t * 64 + lane];
      const u32x4_t a1 = wlds[j][1][t * 64 + lane];
#pragma unroll
      for (int mb = 0; mb < MBW; ++mb) {
        a[0][mb] = mfma_f16(a0, xr[jx][mb][t], a[0][mb]);
        a[1][mb] = mfma_f16(a1, xr[jx][mb][t], a[1][mb]);
      }
    }
#pragma unroll
    for (int mb = 0; mb < MBW; ++mb)
#pragma unroll
      for (int t = 0; t < 4; ++t) xr[jx][mb][t] = xb[mb][(size_t)kb_of(i + XS) * 256 + t * 64];
  };
  auto quarter = [&](f32x16_t (&a)[2][MBW], int q) __attribute__((always_inline)) {
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int mb = 0; mb < MBW; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) a[nb][mb][r] = 0.f;
    for (int i = q * kb_per_quarter; i < (q + 1) * kb_per_quarter; i += 4) {
      iter(a, i, std::integral_constant<int, 0>{});
      iter(a, i + 1, std::integral_constant<int, 1>{});
      iter(a, i + 2, std::integral_constant<int, 2>{});
      iter(a, i + 3, std::integral_constant<int, 3>{});
    }
  };
  f32x16_t acc[2][MBW], other[2][MBW];
  quarter(acc, 0);
  for (int q = 1; q < 4; ++q) {
    quarter(other, q);
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int mb = 0; mb < MBW; ++mb) acc[nb][mb] += other[nb][mb];
  }

  if (!has_rows) return;
  const int col = lane & 31, hb = lane >> 5;
#pragma unroll
  for (int mb = 0; mb < MBW; ++mb) {
    const int m = (m_blk0 + mb) * 32 + col;
    if (m >= M) continue;
    float sum[2][16];
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int r = 0; r < 16; ++r) sum[nb][r] = acc[nb][mb][r];
    store_block<EPI>(sum, m, hb, rb0, rb1, blockIdx.y, M, N, out, se, blockIdx.x);
  }
}

// Wide tile for batches of 65..256 rows: the block owns RBN 32-row blocks of the weight matrix (128 rows, or 96 where
// that makes the tiles as many as the compute units) and the four waves split the batch columns, 32*MBW each.  What
// every block must pull through L2 per k block is its weight tile plus the whole activation panel, and with 64-row
// tiles the panel re-reads (one per block) are 2-4x the weight stream: the projection is then bound by what the L2 can
// deliver, not by HBM.  A larger tile means fewer blocks and with them less panel traffic.  A block runs one wave per
// SIMD and its steps (stage, barrier, multiply) do not overlap, so the time of a launch follows the steps of its
// longest-running compute unit: 256 tiles of 96 rows finish sooner than 192 tiles of 128 rows that leave 64 units idle.
// Same K quarters, same order inside a quarter, quarters added in order: same bits.
template <int MBW, int EPI, int XS, int RBN>
__global__ __launch_bounds__(256, RBN == 3 ? 1 : 2) void gemm_bf16_lds4_kernel(const u32x4_t* __restrict__ X, const u32x4_t* __restrict__ W,
                                                              void* __restrict__ out, int M, int N, int K,
                                                              int kb_per_quarter, int tiles_x, SampleEpilogue se) {
  static_assert(RBN == 4 || (RBN == 3 && EPI != kEpiSample), "the sampling epilogue works on pairs of row blocks");
  __shared__ u32x4_t wlds[4][RBN][256];  // four stages x RBN row blocks x 4 KiB
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int KB = K >> 6;
  const int n_blocks_m = (M + 31) >> 5;
  // Two batch tiles (gridDim.z == 2 is folded into x by the launcher: tiles_x > 0): the two blocks of a weight tile
  // get x indices 8 apart, so they land on the same die at about the same time and share the weights in its L2.
  int tile_x = blockIdx.x, m_tile = blockIdx.z;
  if (tiles_x > 0) {
    const int grp = blockIdx.x >> 4, r = blockIdx.x & 15;
    m_tile = r >> 3;
    tile_x = grp * 8 + (r & 7);
  }
  const int m_blk0 = (m_tile * 4 + wave) * MBW;
  const bool has_rows = m_blk0 < n_blocks_m;

  // row blocks of the tile; those past the end of the matrix shadow its last one (computed, never stored)
  const int n_rb = EPI == kEpiSwiGLU ? (N >> 4) : (N >> 5);
  int rb[RBN];
#pragma unroll
  for (int b = 0; b < RBN; ++b) rb[b] = min(tile_x * RBN + b, n_rb - 1);
  const u32x4_t* wp[RBN];
#pragma unroll
  for (int b = 0; b < RBN; ++b) wp[b] = W + (size_t)rb[b] * KB * 256 + tid;
  const u32x4_t* xb[MBW];
#pragma unroll
  for (int mb = 0; mb < MBW; ++mb) {
    int blk = m_blk0 + mb;
    if (blk >= n_blocks_m) blk = n_blocks_m - 1;  // idle waves and surplus blocks shadow a valid one (never stored)
    xb[mb] = X + (size_t)blk * KB * 256 + lane;
  }
  const int n = 4 * kb_per_quarter;
  const int kb0 = blockIdx.y * n;
  auto kb_of = [&](int i) { return kb0 + (i < n ? i : n - 1); };  // clamped: no conditional loads in the pipeline
  // Weight k blocks are loaded strictly in order (0, 1, 2, ...; the last one again once the range is exhausted), so
  // the slot of the next one is kept as (block within its quarter, quarter) and stepped, without a division.
  int w_r = 0, w_q = 0;
  auto next_wslot = [&]() {
    const int off = (((int)blockIdx.y * kb_per_quarter + w_r) * 4 + w_q) * 256;
    if (w_r + 1 < kb_per_quarter) ++w_r;
    else if (w_q < 3) { w_r = 0; ++w_q; }
    return off;
  };

  u32x4_t wr[4][RBN];        // weight registers: slot s holds a k block with index = s (mod 4)
  u32x4_t xr[XS][MBW][4];    // activation fragments: slot s holds a k block with index = s (mod XS)
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const int ow = next_wslot();
#pragma unroll
    for (int b = 0; b < RBN; ++b) wr[s][b] = __builtin_nontemporal_load(wp[b] + ow);
  }
#pragma unroll
  for (int s = 0; s < XS; ++s)
#pragma unroll
    for (int mb = 0; mb < MBW; ++mb)
#pragma unroll
      for (int t = 0; t < 4; ++t) xr[s][mb][t] = xb[mb][(size_t)kb_of(s) * 256 + t * 64];
  {
    const int ow = next_wslot();
#pragma unroll
    for (int b = 0; b < RBN; ++b) {
      wlds[0][b][tid] = wr[0][b];
      wr[0][b] = __builtin_nontemporal_load(wp[b] + ow);
    }
  }

  auto iter = [&](f32x16_t (&a)[RBN][MBW], int i, auto jc) __attribute__((always_inline)) {
    constexpr int j = decltype(jc)::value, jn = (j + 1) & 3, jx = j % XS;
    const int ow = next_wslot();  // k block i + 5
#pragma unroll
    for (int b = 0; b < RBN; ++b) {
      wlds[jn][b][tid] = wr[jn][b];
      wr[jn][b] = __builtin_nontemporal_load(wp[b] + ow);
    }
    // barrier that orders LDS traffic only (a full one would drain the global loads in flight)
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
#pragma unroll
    for (int t = 0; t < 4; ++t) {
#pragma unroll
      for (int b = 0; b < RBN; ++b) {
        const u32x4_t afrag = wlds[j][b][t * 64 + lane];
#pragma unroll
        for (int mb = 0; mb < MBW; ++mb) a[b][mb] = mfma_f16(afrag, xr[jx][mb][t], a[b][mb]);
      }
    }
#pragma unroll
    for (int mb = 0; mb < MBW; ++mb)
#pragma unroll
      for (int t = 0; t < 4; ++t) xr[jx][mb][t] = xb[mb][(size_t)kb_of(i + XS) * 256 + t * 64];
  };
  auto quarter = [&](f32x16_t (&a)[RBN][MBW], int q) __attribute__((always_inline)) {
#pragma unroll
    for (int b = 0; b < RBN; ++b)
#pragma unroll
      for (int mb = 0; mb < MBW; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) a[b][mb][r] = 0.f;
    for (int i = q * kb_per_quarter; i < (q + 1) * kb_per_quarter; i += 4) {
      iter(a, i, std::integral_constant<int, 0>{});
      iter(a, i + 1, std::integral_constant<int, 1>{});
      iter(a, i + 2, std::integral_constant<int, 2>{});
      iter(a, i + 3, std::integral_constant<int, 3>{});
    }
  };
  f32x16_t acc[RBN][MBW], other[RBN][MBW];
  quarter(acc, 0);
  for (int q = 1; q < 4; ++q) {
    quarter(other, q);
#pragma unroll
    for (int b = 0; b < RBN; ++b)
#pragma unroll
      for (int mb = 0; mb < MBW; ++mb) acc[b][mb] += other[b][mb];
  }

  if (!has_rows) return;
  const int col = lane & 31, hb = lane >> 5;
#pragma unroll
  for (int mb = 0; mb < MBW; ++mb) {
    const int m = (m_blk0 + mb) * 32 + col;
    if (m >= M) continue;
    if constexpr (RBN == 4) {  // as two 64-row tiles (the sampling epilogue works per tile)
#pragma unroll
      for (int p = 0; p < 2; ++p) {
        if (tile_x * 4 + 2 * p >= n_rb) break;
        float sum[2][16];
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
          for (int r = 0; r < 16; ++r) sum[nb][r] = acc[2 * p + nb][mb][r];
        store_block<EPI>(sum, m, hb, rb[2 * p], rb[2 * p + 1], blockIdx.y, M, N, out, se, tile_x * 2 + p);
      }
    } else {
#pragma unroll
      for (int b = 0; b < RBN; ++b) {
        if (tile_x * RBN + b >= n_rb) break;
        float sum[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) sum[r] = acc[b][mb][r];
        store_rowblock<EPI>(sum, m, hb, rb[b], blockIdx.y, M, N, out);
      }
    }
  }
}

// The same tile with eight waves for 129..256 rows: one block holds a 128-row weight tile and all (up to) 256 batch
// rows, 32 per wave, so the weight tile is staged once for both halves of the batch and a compute unit never holds
// two blocks' worth of panel traffic while its neighbour holds one.  Each half of the block stages two of the four
// row blocks.  Same K quarters, same order: same bits.
template <int EPI, int XS>
__global__ __launch_bounds__(512, 1) void gemm_bf16_lds8_kernel(const u32x4_t* __restrict__ X, const u32x4_t* __restrict__ W,
                                                              void* __restrict__ out, int M, int N, int K,
                                                              int kb_per_quarter, SampleEpilogue se) {
  constexpr int MBW = 1;
  __shared__ u32x4_t wlds[4][4][256];  // four stages x four row blocks x 4 KiB
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int KB = K >> 6;
  const int n_blocks_m = (M + 31) >> 5;
  const int half = tid >> 8, t256 = tid & 255;  // which pair of row blocks this thread stages, and where in them
  const int tile_x = blockIdx.x;
  const int m_blk0 = blockIdx.z * 8 + wave;
  const bool has_rows = m_blk0 < n_blocks_m;

  // row blocks: pair p = 64-row tile 2x + p (the second pair shadows the first when the tile count is odd)
  const int n_tiles = EPI == kEpiSwiGLU ? (N >> 5) : (N >> 6);
  int tile[2], rb[4];
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    tile[p] = min(tile_x * 2 + p, n_tiles - 1);
    rb[2 * p] = tile[p] * 2;
    rb[2 * p + 1] = tile[p] * 2 + 1;
  }
  const bool second_valid = tile_x * 2 + 1 < n_tiles;
  const u32x4_t* wp[2];
#pragma unroll
  for (int b = 0; b < 2; ++b) wp[b] = W + (size_t)rb[2 * half + b] * KB * 256 + t256;
  const u32x4_t* xb[MBW];
#pragma unroll
  for (int mb = 0; mb < MBW; ++mb) {
    int blk = m_blk0 + mb;
    if (blk >= n_blocks_m) blk = n_blocks_m - 1;  // idle waves and surplus blocks shadow a valid one (never stored)
    xb[mb] = X + (size_t)blk * KB * 256 + lane;
  }
  const int n = 4 * kb_per_quarter;
  const int kb0 = blockIdx.y * n;
  auto kb_of = [&](int i) { return kb0 + (i < n ? i : n - 1); };  // clamped: no conditional loads in the pipeline
  // Weight k blocks are loaded strictly in order (0, 1, 2, ...; the last one again once the range is exhausted), so
  // the slot of the next one is kept as (block within its quarter, quarter) and stepped, without a division.
  int w_r = 0, w_q = 0;
  auto next_wslot = [&]() {
    const int off = (((int)blockIdx.y * kb_per_quarter + w_r) * 4 + w_q) * 256;
    if (w_r + 1 < kb_per_quarter) ++w_r;
    else if (w_q < 3) { w_r = 0; ++w_q; }
    return off;
  };

  u32x4_t wr[4][2];          // weight registers: slot s holds a k block with index = s (mod 4)
  u32x4_t xr[XS][MBW][4];    // activation fragments: slot s holds a k block with index = s (mod XS)
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const int ow = next_wslot();
#pragma unroll
    for (int b = 0; b < 2; ++b) wr[s][b] = __builtin_nontemporal_load(wp[b] + ow);
  }
#pragma unroll
  for (int s = 0; s < XS; ++s)
#pragma unroll
    for (int mb = 0; mb < MBW; ++mb)
#pragma unroll
      for (int t = 0; t < 4; ++t) xr[s][mb][t] = xb[mb][(size_t)kb_of(s) * 256 + t * 64];
  {
    const int ow = next_wslot();
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      wlds[0][2 * half + b][t256] = wr[0][b];
      wr[0][b] = __builtin_nontemporal_load(wp[b] + ow);
    }
  }

  auto iter = [&](f32x16_t (&a)[4][MBW], int i, auto jc) __attribute__((always_inline)) {
    constexpr int j = decltype(jc)::value, jn = (j + 1) & 3, jx = j % XS;
    const int ow = next_wslot();  // k block i + 5
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      wlds[jn][2 * half + b][t256] = wr[jn][b];
      wr[jn][b] = __builtin_nontemporal_load(wp[b] + ow);
    }
    // barrier that orders LDS traffic only (a full one would drain the global loads in flight)
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
#pragma unroll
    for (int t = 0; t < 4; ++t) {
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const u32x4_t afrag = wlds[j][b][t * 64 + lane];
#pragma unroll
        for (int mb = 0; mb < MBW; ++mb) a[b][mb] = mfma_f16(afrag, xr[jx][mb][t], a[b][mb]);
      }
    }
#pragma unroll
    for (int mb = 0; mb < MBW; ++mb)
#pragma unroll
      for (int t = 0; t < 4; ++t) xr[jx][mb][t] = xb[mb][(size_t)kb_of(i + XS) * 256 + t * 64];
  };
  auto quarter = [&](f32x16_t (&a)[4][MBW], int q) __attribute__((always_inline)) {
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int mb = 0; mb < MBW; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) a[b][mb][r] = 0.f;
    for (int i = q * kb_per_quarter; i < (q + 1) * kb_per_quarter; i += 4) {
      iter(a, i, std::integral_constant<int, 0>{});
      iter(a, i + 1, std::integral_constant<int, 1>{});
      iter(a, i + 2, std::integral_constant<int, 2>{});
      iter(a, i + 3, std::integral_constant<int, 3>{});
    }
  };
  f32x16_t acc[4][MBW], other[4][MBW];
  quarter(acc, 0);
  for (int q = 1; q < 4; ++q) {
    quarter(other, q);
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int mb = 0; mb < MBW; ++mb) acc[b][mb] += other[b][mb];
  }

  if (!has_rows) return;
  const int col = lane & 31, hb = lane >> 5;
#pragma unroll
  for (int mb = 0; mb < MBW; ++mb) {
    const int m = (m_blk0 + mb) * 32 + col;
    if (m >= M) continue;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      if (p == 1 && !second_valid) break;
      float sum[2][16];
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r) sum[nb][r] = acc[2 * p + nb][mb][r];
      store_block<EPI>(sum, m, hb, rb[2 * p], rb[2 * p + 1], blockIdx.y, M, N, out, se, tile[p]);
    }
  }
}

// The eight-wave block with a 96-row weight tile (three row blocks), for matrices whose 128-row tiles would leave a
// quarter of the compute units without a block while 96-row tiles give every unit one.  The first four waves stage
// row blocks 0 and 2, the other four row block 1; each half runs its own copy of the loop (same steps, one barrier
// per k block in both), so that no load in the pipeline is conditional.  Same K quarters, same order: same bits.
template <int EPI, int XS>
__global__ __launch_bounds__(512, 1) void gemm_bf16_lds8r3_kernel(const u32x4_t* __restrict__ X, const u32x4_t* __restrict__ W,
                                                                void* __restrict__ out, int M, int N, int K,
                                                                int kb_per_quarter) {
  static_assert(EPI != kEpiSample, "per-row-block epilogues only");
  constexpr int MBW = 1, RBN = 3;
  __shared__ u32x4_t wlds[4][RBN][256];  // four stages x three row blocks x 4 KiB
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int KB = K >> 6;
  const int n_blocks_m = (M + 31) >> 5;
  const int t256 = tid & 255;
  const int tile_x = blockIdx.x;
  const int m_blk0 = blockIdx.z * 8 + wave;
  const bool has_rows = m_blk0 < n_blocks_m;
  const int n_rb = EPI == kEpiSwiGLU ? (N >> 4) : (N >> 5);
  int rb[RBN];
#pragma unroll
  for (int b = 0; b < RBN; ++b) rb[b] = min(tile_x * RBN + b, n_rb - 1);  // past the end: shadows the last one, never stored
  const u32x4_t* xb[MBW];
#pragma unroll
  for (int mb = 0; mb < MBW; ++mb) {
    int blk = m_blk0 + mb;
    if (blk >= n_blocks_m) blk = n_blocks_m - 1;  // idle waves shadow a valid block (never stored)
    xb[mb] = X + (size_t)blk * KB * 256 + lane;
  }
  const int n = 4 * kb_per_quarter;
  const int kb0 = blockIdx.y * n;
  auto kb_of = [&](int i) { return kb0 + (i < n ? i : n - 1); };  // clamped: no conditional loads in the pipeline
  f32x16_t acc[RBN][MBW];

  // NS = row blocks this half of the block stages: srb[0 .. NS-1]
  auto run = [&](auto ns_c, int srb0, int srb1) __attribute__((always_inline)) {
    constexpr int NS = decltype(ns_c)::value;
    const int srb[2] = {srb0, srb1};
    const u32x4_t* wp[NS];
#pragma unroll
    for (int b = 0; b < NS; ++b) wp[b] = W + (size_t)rb[srb[b]] * KB * 256 + t256;
    // Weight k blocks are loaded strictly in order (the last one again once the range is exhausted); the slot of the
    // next one is kept as (block within its quarter, quarter) and stepped, without a division.
    int w_r = 0, w_q = 0;
    auto next_wslot = [&]() {
      const int off = (((int)blockIdx.y * kb_per_quarter + w_r) * 4 + w_q) * 256;
      if (w_r + 1 < kb_per_quarter) ++w_r;
      else if (w_q < 3) { w_r = 0; ++w_q; }
      return off;
    };
    u32x4_t wr[4][NS];        // weight registers: slot s holds a k block with index = s (mod 4)
    u32x4_t xr[XS][MBW][4];   // activation fragments: slot s holds a k block with index = s (mod XS)
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const int ow = next_wslot();
#pragma unroll
      for (int b = 0; b < NS; ++b) wr[s][b] = __builtin_nontemporal_load(wp[b] + ow);
    }
#pragma unroll
    for (int s = 0; s < XS; ++s)
#pragma unroll
      for (int mb = 0; mb < MBW; ++mb)
#pragma unroll
        for (int t = 0; t < 4; ++t) xr[s][mb][t] = xb[mb][(size_t)kb_of(s) * 256 + t * 64];
    {
      const int ow = next_wslot();
#pragma unroll
      for (int b = 0; b < NS; ++b) {
        wlds[0][srb[b]][t256] = wr[0][b];
        wr[0][b] = __builtin_nontemporal_load(wp[b] + ow);
      }
    }
    auto iter = [&](f32x16_t (&a)[RBN][MBW], int i, auto jc) __attribute__((always_inline)) {
      constexpr int j = decltype(jc)::value, jn = (j + 1) & 3, jx = j % XS;
      const int ow = next_wslot();  // k block i + 5
#pragma unroll
      for (int b = 0; b < NS; ++b) {
        wlds[jn][srb[b]][t256] = wr[jn][b];
        wr[jn][b] = __builtin_nontemporal_load(wp[b] + ow);
      }
      // barrier that orders LDS traffic only (a full one would drain the global loads in flight)
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
      __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
#pragma unroll
      for (int t = 0; t < 4; ++t) {
#pragma unroll
        for (int b = 0; b < RBN; ++b) {
          const u32x4_t afrag = wlds[j][b][t * 64 + lane];
#pragma unroll
          for (int mb = 0; mb < MBW; ++mb) a[b][mb] = mfma_f16(afrag, xr[jx][mb][t], a[b][mb]);
        }
      }
#pragma unroll
      for (int mb = 0; mb < MBW; ++mb)
#pragma unroll
        for (int t = 0; t < 4; ++t) xr[jx][mb][t] = xb[mb][(size_t)kb_of(i + XS) * 256 + t * 64];
    };
    auto quarter = [&](f32x16_t (&a)[RBN][MBW], int q) __attribute__((always_inline)) {
#pragma unroll
      for (int b = 0; b < RBN; ++b)
#pragma unroll
        for (int mb = 0; mb < MBW; ++mb)
#pragma unroll
          for (int r = 0; r < 16; ++r) a[b][mb][r] = 0.f;
      for (int i = q * kb_per_quarter; i < (q + 1) * kb_per_quarter; i += 4) {
        iter(a, i, std::integral_constant<int, 0>{});
        iter(a, i + 1, std::integral_constant<int, 1>{});
        iter(a, i + 2, std::integral_constant<int, 2>{});
        iter(a, i + 3, std::integral_constant<int, 3>{});
      }
    };
    f32x16_t other[RBN][MBW];
    quarter(acc, 0);
    for (int q = 1; q < 4; ++q) {
      quarter(other, q);
#pragma unroll
      for (int b = 0; b < RBN; ++b)
#pragma unroll
        for (int mb = 0; mb < MBW; ++mb) acc[b][mb] += other[b][mb];
    }
  };
  if (__builtin_amdgcn_readfirstlane(wave) < 4) run(std::integral_constant<int, 2>{}, 0, 2);
  else run(std::integral_constant<int, 1>{}, 1, 1);

  if (!has_rows) return;
  const int col = lane & 31, hb = lane >> 5;
#pragma unroll
  for (int mb = 0; mb < MBW; ++mb) {
    const int m = (m_blk0 + mb) * 32 + col;
    if (m >= M) continue;
#pragma unroll
    for (int b = 0; b < RBN; ++b) {
      if (tile_x * RBN + b >= n_rb) break;
      float sum[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) sum[r] = acc[b][mb][r];
      store_rowblock<EPI>(sum, m, hb, rb[b], blockIdx.y, M, N, out);
    }
  }
}

struct Plan {
  int splits;       // K splits across blocks
  int kb_per_wave;  // 64-wide k blocks per wave
};

Plan make_plan(int N, int K, int epi, bool allow_split) {
  const int KB = K >> 6;
  const int tiles = epi == kEpiSwiGLU ? (N >> 5) : (N >> 6);
  int S = 1;
  // Split K across blocks until about one block per CU exists; each wave keeps >= 2 k blocks.
  while (tiles * S < 256 && (KB % (S * 2 * 4) == 0) && KB / (S * 2 * 4) >= 2 && epi == kEpiPartial && allow_split) S *= 2;
  return Plan{S, KB / (S * 4)};
}

template <int MB, int ST>
void launch_mb(hipStream_t s, const void* X, const void* W, void* out, int M, int N, int K, int epi, bool allow_split,
               const SampleEpilogue& se) {
  Plan p = make_plan(N, K, epi, allow_split);
  const int m_tiles = (M + 32 * MB - 1) / (32 * MB);
  if (epi == kEpiSwiGLU) {
    dim3 grid(N >> 5, 1, m_tiles);
    gemm_bf16_kernel<MB, kEpiSwiGLU, ST><<<grid, 256, 0, s>>>((const u32x4_t*)X, (const u32x4_t*)W, out, M, N, K, p.kb_per_wave, se);
  } else if (epi == kEpiSample) {
    dim3 grid(N >> 6, 1, m_tiles);
    gemm_bf16_kernel<MB, kEpiSample, ST><<<grid, 256, 0, s>>>((const u32x4_t*)X, (const u32x4_t*)W, out, M, N, K, p.kb_per_wave, se);
  } else {
    dim3 grid(N >> 6, p.splits, m_tiles);
    gemm_bf16_kernel<MB, kEpiPartial, ST><<<grid, 256, 0, s>>>((const u32x4_t*)X, (const u32x4_t*)W, out, M, N, K, p.kb_per_wave, se);
  }
}

template <int MB, int ST>
void launch_wide(hipStream_t s, const void* X, const void* W, void* out, int M, int N, int K, int epi, bool allow_split,
                 const SampleEpilogue& se) {
  Plan p = make_plan(N, K, epi, allow_split);  // same K split as the narrow tiling: bit-identical results
  const int m_tiles = (M + 32 * MB - 1) / (32 * MB);
  const int tiles = epi == kEpiSwiGLU ? (N >> 5) : (N >> 6);
  dim3 grid((tiles + 1) / 2, epi == kEpiPartial ? p.splits : 1, m_tiles);
  if (epi == kEpiSwiGLU)
    gemm_bf16_wide_kernel<MB, kEpiSwiGLU, ST><<<grid, 256, 0, s>>>((const u32x4_t*)X, (const u32x4_t*)W, out, M, N, K, p.kb_per_wave, se);
  else if (epi == kEpiSample)
    gemm_bf16_wide_kernel<MB, kEpiSample, ST><<<grid, 256, 0, s>>>((const u32x4_t*)X, (const u32x4_t*)W, out, M, N, K, p.kb_per_wave, se);
  else
    gemm_bf16_wide_kernel<MB, kEpiPartial, ST><<<grid, 256, 0, s>>>((const u32x4_t*)X, (const u32x4_t*)W, out, M, N, K, p.kb_per_wave, se);
}

// Tiles of two sizes (see gemm_bf16_mixed_kernel): used when the matrix has exactly three (row block, K split) units
// per compute unit.
constexpr int kComputeUnits = 256;
bool mixed_fits(int N, int K, int epi, bool allow_split) {
  if (epi == kEpiSample) return false;
  const Plan p = make_plan(N, K, epi, allow_split);
  const int row_blocks = (epi == kEpiSwiGLU ? 2 * N : N) >> 5;
  return row_blocks % 3 == 0 && row_blocks * p.splits == 3 * kComputeUnits;
}

template <int MB, int ST>
void launch_mixed(hipStream_t s, const void* X, const void* W, void* out, int M, int N, int K, int epi, bool allow_split,
                  const SampleEpilogue& se) {
  const Plan p = make_plan(N, K, epi, allow_split);  // same K split as the other variants: bit-identical results
  const int row_blocks = (epi == kEpiSwiGLU ? 2 * N : N) >> 5, third = row_blocks / 3;
  const int m_tiles = (M + 32 * MB - 1) / (32 * MB);
  dim3 grid(p.splits * 2 * third, 1, m_tiles);
  if (epi == kEpiSwiGLU)
    gemm_bf16_mixed_kernel<MB, kEpiSwiGLU, ST><<<grid, 256, 0, s>>>((const u32x4_t*)X, (const u32x4_t*)W, out, M, N, K,
                                                                    p.kb_per_wave, third, third, p.splits, se);
  else
    gemm_bf16_mixed_kernel<MB, kEpiPartial, ST><<<grid, 256, 0, s>>>((const u32x4_t*)X, (const u32x4_t*)W, out, M, N, K,
                                                                     p.kb_per_wave, third, third, p.splits, se);
}

// Blocks of the 128-row tiling for (N, K): it is used where they still fill the chip.
int wide_blocks(int N, int K, int epi, bool allow_split) {
  const Plan p = make_plan(N, K, epi, allow_split);
  const int tiles = epi == kEpiSwiGLU ? (N >> 5) : (N >> 6);
  return ((tiles + 1) / 2) * (epi == kEpiPartial ? p.splits : 1);
}

}  // namespace

int gemm_bf16_splits(int N, int K, int epi) { return make_plan(N, K, epi, true).splits; }
int gemm_bf16_weight_segment(int N, int K, bool split_k) { return make_plan(N, K, kEpiPartial, split_k).kb_per_wave; }

template <int MB>
void launch_st(hipStream_t s, const void* X, const void* W, void* out, int M, int N, int K, int epi, bool allow_split,
               int stages, const SampleEpilogue& se) {
  const int n = make_plan(N, K, epi, allow_split).kb_per_wave;
  if (stages > n) stages = n;  // the kernel's prologue fills all of its buffers unconditionally
  switch (stages) {
    case 1: launch_mb<MB, 1>(s, X, W, out, M, N, K, epi, allow_split, se); break;
    case 2: launch_mb<MB, 2>(s, X, W, out, M, N, K, epi, allow_split, se); break;
    case 3: launch_mb<MB, 3>(s, X, W, out, M, N, K, epi, allow_split, se); break;
    default: launch_mb<MB, 4>(s, X, W, out, M, N, K, epi, allow_split, se); break;
  }
}

template <int MBW, int ST>
void launch_cols_st(hipStream_t s, const void* X, const void* W, void* out, int M, int N, int K, int epi, bool allow_split,
                    const SampleEpilogue& se) {
  Plan p = make_plan(N, K, epi, allow_split);  // same K split as the other variants: bit-identical results
  const int m_tiles = (M + 128 * MBW - 1) / (128 * MBW);
  if (epi == kEpiSwiGLU) {
    dim3 grid(N >> 5, 1, m_tiles);
    gemm_bf16_cols_kernel<MBW, kEpiSwiGLU, ST><<<grid, 256, 0, s>>>((const u32x4_t*)X, (const u32x4_t*)W, out, M, N, K, p.kb_per_wave, se);
  } else if (epi == kEpiSample) {
    dim3 grid(N >> 6, 1, m_tiles);
    gemm_bf16_cols_kernel<MBW, kEpiSample, ST><<<grid, 256, 0, s>>>((const u32x4_t*)X, (const u32x4_t*)W, out, M, N, K, p.kb_per_wave, se);
  } else {
    dim3 grid(N >> 6, p.splits, m_tiles);
    gemm_bf16_cols_kernel<MBW, kEpiPartial, ST><<<grid, 256, 0, s>>>((const u32x4_t*)X, (const u32x4_t*)W, out, M, N, K, p.kb_per_wave, se);
  }
}

template <int MBW, int XS>
void launch_lds(hipStream_t s, const void* X, const void* W, void* out, int M, int N, int K, int epi, bool allow_split,
                const SampleEpilogue& se) {
  Plan p = make_plan(N, K, epi, allow_split);
  const int m_tiles = (M + 128 * MBW - 1) / (128 * MBW);
  if (epi == kEpiSwiGLU) {
    dim3 grid(N >> 5, 1, m_tiles);
    gemm_bf16_lds_kernel<MBW, kEpiSwiGLU, XS><<<grid, 256, 0, s>>>((const u32x4_t*)X, (const u32x4_t*)W, out, M, N, K, p.kb_per_wave, se);
  } else if (epi == kEpiSample) {
    dim3 grid(N >> 6, 1, m_tiles);
    gemm_bf16_lds_kernel<MBW, kEpiSample, XS><<<grid, 256, 0, s>>>((const u32x4_t*)X, (const u32x4_t*)W, out, M, N, K, p.kb_per_wave, se);
  } else {
    dim3 grid(N >> 6, p.splits, m_tiles);
    gemm_bf16_lds_kernel<MBW, kEpiPartial, XS><<<grid, 256, 0, s>>>((const u32x4_t*)X, (const u32x4_t*)W, out, M, N, K, p.kb_per_wave, se);
  }
}

template <int MBW, int XS, int RBN = 4>
void launch_lds4(hipStream_t s, const void* X, const void* W, void* out, int M, int N, int K, int epi, bool allow_split,
                 const SampleEpilogue& se) {
  Plan p = make_plan(N, K, epi, allow_split);  // same K split as the other variants: bit-identical results
  const int m_tiles = (M + 128 * MBW - 1) / (128 * MBW);
  const int n_rb = epi == kEpiSwiGLU ? (N >> 4) : (N >> 5);
  const int tx = (n_rb + RBN - 1) / RBN;
  const bool fold = m_tiles == 2 && (tx & 7) == 0;  // pair the two batch tiles of a weight tile on one die
  dim3 grid(fold ? 2 * tx : tx, epi == kEpiPartial ? p.splits : 1, fold ? 1 : m_tiles);
  const int tiles_x = fold ? tx : 0;
  if (epi == kEpiSwiGLU)
    gemm_bf16_lds4_kernel<MBW, kEpiSwiGLU, XS, RBN><<<grid, 256, 0, s>>>((const u32x4_t*)X, (const u32x4_t*)W, out, M, N, K, p.kb_per_wave, tiles_x, se);
  else if (epi == kEpiSample) {
    if constexpr (RBN == 4)
      gemm_bf16_lds4_kernel<MBW, kEpiSample, XS, 4><<<grid, 256, 0, s>>>((const u32x4_t*)X, (const u32x4_t*)W, out, M, N, K, p.kb_per_wave, tiles_x, se);
  } else
    gemm_bf16_lds4_kernel<MBW, kEpiPartial, XS, RBN><<<grid, 256, 0, s>>>((const u32x4_t*)X, (const u32x4_t*)W, out, M, N, K, p.kb_per_wave, tiles_x, se);
}

void launch_lds8(hipStream_t s, const void* X, const void* W, void* out, int M, int N, int K, int epi, bool allow_split,
                 const SampleEpilogue& se) {
  Plan p = make_plan(N, K, epi, allow_split);  // same K split as the other variants: bit-identical results
  const int tiles = epi == kEpiSwiGLU ? (N >> 5) : (N >> 6);
  dim3 grid((tiles + 1) / 2, epi == kEpiPartial ? p.splits : 1, (M + 255) / 256);
  if (epi == kEpiSwiGLU)
    gemm_bf16_lds8_kernel<kEpiSwiGLU, 2><<<grid, 512, 0, s>>>((const u32x4_t*)X, (const u32x4_t*)W, out, M, N, K, p.kb_per_wave, se);
  else if (epi == kEpiSample)
    gemm_bf16_lds8_kernel<kEpiSample, 2><<<grid, 512, 0, s>>>((const u32x4_t*)X, (const u32x4_t*)W, out, M, N, K, p.kb_per_wave, se);
  else
    gemm_bf16_lds8_kernel<kEpiPartial, 2><<<grid, 512, 0, s>>>((const u32x4_t*)X, (const u32x4_t*)W, out, M, N, K, p.kb_per_wave, se);
}

template <int MBW>
void launch_cols(hipStream_t s, const void* X, const void* W, void* out, int M, int N, int K, int epi, bool allow_split,
                 const SampleEpilogue& se) {
  if (make_plan(N, K, epi, allow_split).kb_per_wave % 4 == 0) {  // weight tiles shared through LDS
    // The wide tile pays where it still leaves enough blocks to fill the chip.
    const Plan p = make_plan(N, K, epi, allow_split);
    const int tiles = epi == kEpiSwiGLU ? (N >> 5) : (N >> 6);
    const int wide_blocks = ((tiles + 1) / 2) * (epi == kEpiPartial ? p.splits : 1);
    // 129..256 rows: one block of eight waves per weight tile where that still gives >= 192 blocks (gate/up 82 -> 65 us,
    // QKV 33 -> 29, output projection 538 -> 420 at 256 rows); the O and down projections would be left with 128 blocks
    // (measured 21 -> 26 and 42 -> 50 us) and run as two batch tiles of 128 whose blocks are paired on one die.
    // (more than 256 rows: the batch tiles of 256 count as blocks too, which brings the O and down projections in)
    if (M > 128 && wide_blocks * ((M + 255) / 256) >= 192) {
      // ... and 96-row tiles where those give every compute unit a block and 128-row tiles do not (M <= 256: one
      // batch tile per weight tile; gate/up and QKV of the 8B shape)
      const int n_rb = epi == kEpiSwiGLU ? (N >> 4) : (N >> 5);
      const int splits = epi == kEpiPartial ? p.splits : 1;
      if (M <= 256 && epi != kEpiSample && n_rb % 3 == 0 && wide_blocks < kComputeUnits && (n_rb / 3) * splits <= kComputeUnits) {
        dim3 grid(n_rb / 3, splits, 1);
        if (epi == kEpiSwiGLU)
          gemm_bf16_lds8r3_kernel<kEpiSwiGLU, 2><<<grid, 512, 0, s>>>((const u32x4_t*)X, (const u32x4_t*)W, out, M, N, K, p.kb_per_wave);
        else
          gemm_bf16_lds8r3_kernel<kEpiPartial, 2><<<grid, 512, 0, s>>>((const u32x4_t*)X, (const u32x4_t*)W, out, M, N, K, p.kb_per_wave);
        return;
      }
      launch_lds8(s, X, W, out, M, N, K, epi, allow_split, se);
      return;
    }
    if (wide_blocks * ((M + 127) / 128) >= 192) {
      // up to 128 rows: 96-row tiles where 128-row tiles would leave a quarter of the compute units without a block
      // and 96-row tiles give every unit one (gate/up 55 -> 41 us, QKV 21 -> 16 us at 128 rows)
      const int n_rb = epi == kEpiSwiGLU ? (N >> 4) : (N >> 5);
      const int splits = epi == kEpiPartial ? p.splits : 1;
      if (M <= 128 && epi != kEpiSample && n_rb % 3 == 0 && wide_blocks < kComputeUnits && (n_rb / 3) * splits <= kComputeUnits) {
        launch_lds4<1, 2, 3>(s, X, W, out, M, N, K, epi, allow_split, se);
        return;
      }
      launch_lds4<1, 2>(s, X, W, out, M, N, K, epi, allow_split, se);
      return;
    }
    launch_lds<MBW, MBW == 1 ? 4 : 2>(s, X, W, out, M, N, K, epi, allow_split, se);
    return;
  }
  // two buffers in flight per wave when the quarter length allows it (it does for every 8B-shaped matrix)
  if (make_plan(N, K, epi, allow_split).kb_per_wave % 2 == 0) launch_cols_st<MBW, 2>(s, X, W, out, M, N, K, epi, allow_split, se);
  else launch_cols_st<MBW, 1>(s, X, W, out, M, N, K, epi, allow_split, se);
}

// Requirements (checked at model init): K % 256 == 0, N % 64 == 0 (N % 32 for SwiGLU).
void launch_gemm_bf16(hipStream_t s, const void* X, const void* W, void* out, int M, int N, int K, int epi,
                      bool allow_split, const SampleEpilogue* se) {
  static const SampleEpilogue none{};
  const SampleEpilogue& e = se ? *se : none;
  if (epi == kEpiSample) allow_split = false;
  // 128-row tiles for the K-split projections whose halved grid still fills the chip (QKV at the 8B shape: 16 -> 15 us
  // at 32 rows, 20.5 -> 17.8 us at 64); measured a loss for gate/up and the output projection, which keep 64-row tiles.
  const bool wide = epi == kEpiPartial && make_plan(N, K, epi, allow_split).splits > 1 &&
                    wide_blocks(N, K, epi, allow_split) >= 192 && make_plan(N, K, epi, allow_split).kb_per_wave >= 2;
  const bool mixed = mixed_fits(N, K, epi, allow_split);
  const int kbw = make_plan(N, K, epi, allow_split).kb_per_wave;
  if (M <= 32 && mixed && kbw >= 4) launch_mixed<1, 4>(s, X, W, out, M, N, K, epi, allow_split, e);
  else if (M <= 64 && M > 32 && mixed && kbw >= 2) launch_mixed<2, 2>(s, X, W, out, M, N, K, epi, allow_split, e);
  else if (M <= 32 && wide) launch_wide<1, 2>(s, X, W, out, M, N, K, epi, allow_split, e);
  else if (M <= 32) launch_st<1>(s, X, W, out, M, N, K, epi, allow_split, 4, e);
  else if (M <= 64 && wide) launch_wide<2, 2>(s, X, W, out, M, N, K, epi, allow_split, e);
  else if (M <= 64) launch_st<2>(s, X, W, out, M, N, K, epi, allow_split, 2, e);
  else if (M <= 128) launch_cols<1>(s, X, W, out, M, N, K, epi, allow_split, e);
  else launch_cols<2>(s, X, W, out, M, N, K, epi, allow_split, e);
}

}  // namespace rl
