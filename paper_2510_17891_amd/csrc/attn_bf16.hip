// GQA decode attention over a paged bf16 KV cache, head_dim 128, split over the context.
//
// The step reads ctx * n_kv * 2 * 256 bytes per row and does ~4 flop per byte: a pure HBM stream.  The kernel
// is therefore built so that every K/V byte is loaded exactly once, with fully coalesced 1 KiB wave loads, straight
// into the registers that feed the matrix cores (the page layouts are chosen for that; see small_kernels.hip):
//
//   scores  S[key][head]  = sum_d K[key][d] q[head][d]   MFMA 16x16x32, A = K page (16 keys), B = q (<= 8 heads
//                                                        of the group, remaining columns zero); q is split into
//                                                        a bf16 high and low part so q keeps ~16 mantissa bits
//   O^T[d][head]          += V^T[d][key] P[key][head]    MFMA 16x16x32 over two pages (32 keys); the P operand is
//                                                        exactly the registers the score MFMA produced
//
// The context is cut into segments whose number and bounds depend on the context length alone
// (4*ceil(ctx/1024) equal runs of 32-key steps), each leaving (max, sum, unnormalised O) per head.  One block of
// four waves handles up to 16 segments of one (row, kv head), each wave a contiguous quarter; beyond 4096 keys a block
// takes `spb` segments (a launch parameter, 4 by default: shorter blocks fill the end of a long launch better).
//   ctx <= 4096: one block per (row, kv head); partials stay in LDS and after a block barrier the four waves
//                merge the segments of one head each, flat and in index order.
//   ctx  > 4096: ceil(segments/spb) blocks per (row, kv head), so that long contexts become many short blocks
//                that the dispatcher can balance; partials go to the workspace and a second small kernel does the
//                same flat merge.
// Which path runs is a function of the row's context only, and nothing synchronises across blocks inside a
// kernel (a device-scope fence is an L2 write-back on this multi-die part), so the bits of a row's result do not
// depend on the batch.
//
// Shared prompt pages (the samples of one prompt, Section 2.3): rows of equal context length whose first pages are
// the same physical pages form sets of up to 16 / group rows, or 32 / group when the launch is large enough to be
// bound by memory traffic.  The same launch holds one more kind of block: a "set" block computes up to four of
// the segments that lie inside the shared pages once for the whole set, the set's (row, head) pairs side by side
// in the columns of the matrix operand (two operands of 16 columns, fed from the same key and value registers,
// for the larger sets).  The rows of a set start after those
// segments; both kinds leave their partials in the workspace and the merge kernel combines them with the
// arithmetic of the in-block merge.  A column of the matrix product does not depend on its neighbours and the
// segment bounds are the same, so a row's bits equal those of the row computed alone.
// Rows that feed neighbouring positions of one sequence (prefill, scoring) form sets in the same way when they lie
// in one aligned window of 32 positions: equal step counts and segments, each row's keys a prefix of the next row's.
// Such a set computes all segments of its rows, every column masked at its own context length, and the window's
// keys are read once per set instead of once per row.
//
// Decode steps (one row per sequence) run the variant that also does what would otherwise be a kernel of its own
// before this one: it sums the QKV projection's split partials, normalises and rotates the heads of its columns, and
// appends the row's new key and value to the cache.  The only consumer of a row's new key and value inside the launch
// is the wave that owns the row's last 32-key step; it gets them from LDS into its operand registers and stores
// them to the page when its work is done, so no wave ever waits for those (small, scattered) stores.
#include <algorithm>
#include <type_traits>

#include "device_utils.h"
#include "kernels.h"
#include "rope_device.h"

namespace rl {

namespace {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

constexpr int kD = 128;
constexpr int kPageElems = kPageTokens * kD;  // 2048 bf16 = 4 KiB per (page, kv head), K or V
constexpr int kPartStride = kD + 2;           // floats per (row, head, segment): O[128], max, sum
// In LDS a segment's record is those 130 floats in a row.  In the workspace the max_segs records of a (row, head) are
// split into the O rows (128 floats each, so that every row is whole cache lines: max_segs is a multiple of 16 and
// with it the 520 * max_segs bytes of a (row, head)) followed by the (max, sum) pairs, which the merge then finds
// side by side.
__device__ __forceinline__ size_t part_o(int max_segs, int seg) { return (size_t)seg * kD; }
__device__ __forceinline__ size_t part_ml(int max_segs, int seg) { return (size_t)max_segs * kD + 2 * (size_t)seg; }
constexpr int kLdsSegs = 16;                  // contexts up to 4096 keep their segment partials in LDS

constexpr int kPairU4(bool kv8) { return kv8 ? 2 * kPageElems / 16 : 2 * kPageElems / 8; }  // 16-byte units of one (page, kv head): K and V

template <bool WRITTEN> struct PoolPtr { typedef const u32x4_t* __restrict__ type; };
template <> struct PoolPtr<true> { typedef const u32x4_t* type; };

struct PagePair {
  u32x4_t k[2][4];  // [page a|b][mfma step s]: keys x dims 32s..32s+31
  u32x4_t v[2][4];  // [page a|b][jj]: dims 32jj..32jj+31 (two 16-dim blocks) x this lane's 4 keys
};

__device__ __forceinline__ void load_pair(PagePair& pp, const u32x4_t* kbase, const u32x4_t* vbase, int64_t page_a,
                                          int64_t page_b, int n_kv, int lane) {
  // per layer the pool is [page][kv head][K | V]: the K and V blocks of a (page, head) are adjacent
  const size_t oa = (size_t)page_a * n_kv * (2 * kPageElems / 8) + lane;
  const size_t ob = (size_t)page_b * n_kv * (2 * kPageElems / 8) + lane;
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    pp.k[0][s] = __builtin_nontemporal_load(kbase + oa + s * 64);
    pp.k[1][s] = __builtin_nontemporal_load(kbase + ob + s * 64);
  }
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    pp.v[0][s] = __builtin_nontemporal_load(vbase + oa + s * 64);
    pp.v[1][s] = __builtin_nontemporal_load(vbase + ob + s * 64);
  }
}

// The same 32 keys from fp8 pages, as loaded: half the registers; widened to a PagePair when the step consumes them.
struct PagePair8 {
  u32x4_t k[2][2];  // [page a|b][c]: this lane's key, dims 64c + 16g .. +15 (two matrix-core steps of 8 dims)
  u32x4_t v[2][2];  // [page a|b][J]: word 2*(jj&1) + par = this lane's 4 keys of dim 32jj + 16par + dl, jj = 2J + (jj&1)
};

__device__ __forceinline__ void load_pair(PagePair8& pp, const u32x4_t* kbase, const u32x4_t* vbase, int64_t page_a,
                                          int64_t page_b, int n_kv, int lane) {
  const size_t oa = (size_t)page_a * n_kv * kPairU4(true) + lane;
  const size_t ob = (size_t)page_b * n_kv * kPairU4(true) + lane;
#pragma unroll
  for (int c = 0; c < 2; ++c) {
    pp.k[0][c] = __builtin_nontemporal_load(kbase + oa + c * 64);
    pp.k[1][c] = __builtin_nontemporal_load(kbase + ob + c * 64);
  }
#pragma unroll
  for (int c = 0; c < 2; ++c) {
    pp.v[0][c] = __builtin_nontemporal_load(vbase + oa + c * 64);
    pp.v[1][c] = __builtin_nontemporal_load(vbase + ob + c * 64);
  }
}

// Four fp8 (one word) -> four bf16 (two words), two values per instruction (the packed conversion with a scale
// operand, scale one); exact, every e4m3 value is a bf16 value.
__device__ __forceinline__ void fp8x4_to_bf16x4(uint32_t w, uint32_t& lo, uint32_t& hi) {
  lo = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, false));
  hi = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, true));
}

__device__ __forceinline__ void widen(PagePair& out, const PagePair8& in) {
#pragma unroll
  for (int p = 0; p < 2; ++p)
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int h = 0; h < 2; ++h) {  // matrix-core step s = 2c + h: dims 64c + 16g + 8h .. +7
        uint32_t w0, w1, w2, w3;
        fp8x4_to_bf16x4(in.k[p][c][2 * h], w0, w1);
        fp8x4_to_bf16x4(in.k[p][c][2 * h + 1], w2, w3);
        out.k[p][2 * c + h] = (u32x4_t){w0, w1, w2, w3};
      }
#pragma unroll
  for (int p = 0; p < 2; ++p)
#pragma unroll
    for (int J = 0; J < 2; ++J)
#pragma unroll
      for (int j2 = 0; j2 < 2; ++j2) {  // jj = 2J + j2: words (par 0: two, par 1: two) as in the bf16 page
        uint32_t w0, w1, w2, w3;
        fp8x4_to_bf16x4(in.v[p][J][2 * j2], w0, w1);
        fp8x4_to_bf16x4(in.v[p][J][2 * j2 + 1], w2, w3);
        out.v[p][2 * J + j2] = (u32x4_t){w0, w1, w2, w3};
      }
}

// Blocks per (row, kv head): contexts of up to kLdsSegs segments take one block (partials merged in LDS), longer ones
// one block per spb segments (spb <= kLdsSegs, a launch parameter: smaller blocks balance better at the end of a
// launch; the partials and their merge do not depend on it).
__host__ __device__ inline int attn_num_splits(int n_seg, int spb) { return n_seg <= kLdsSegs ? 1 : (n_seg + spb - 1) / spb; }

// Flat merge of the (at most kLdsSegs) segments of one head: running maximum, weights exp(m_c - M), sums in index
// order; the lane owns dims 2*lane, 2*lane+1.  o_ptr(c) -> O(128), ml_ptr(c) -> (max, sum) of segment c (LDS or
// workspace); all loads are issued before the arithmetic.  Returns the two normalised outputs packed as f16 (the operand type
// of the output projection).
template <typename F, typename G>
__device__ __forceinline__ uint32_t merge_short(F o_ptr, G ml_ptr, int n_seg, int n_it, int lane) {
  float mx[kLdsSegs], lx[kLdsSegs];
  float2 vx[kLdsSegs];
#pragma unroll
  for (int c = 0; c < kLdsSegs; ++c) {
    mx[c] = -INFINITY;  // marks an absent or empty segment (nothing was written for it)
    lx[c] = 0.f;
    vx[c] = make_float2(0.f, 0.f);
    if (c < n_seg && attn_seg_begin(c + 1, n_it, n_seg) != attn_seg_begin(c, n_it, n_seg)) {
      const float* pm = ml_ptr(c);
      mx[c] = pm[0];
      lx[c] = pm[1];
      vx[c] = *(const float2*)(o_ptr(c) + 2 * lane);
    }
  }
  float M = -INFINITY;
#pragma unroll
  for (int c = 0; c < kLdsSegs; ++c) M = fmaxf(M, mx[c]);
  float o0 = 0.f, o1 = 0.f, den = 0.f;
#pragma unroll
  for (int c = 0; c < kLdsSegs; ++c) {
    if (mx[c] != -INFINITY) {  // a segment with keys has a finite maximum
      const float w = __expf(mx[c] - M);
      den = fmaf(w, lx[c], den);
      o0 = fmaf(w, vx[c].x, o0);
      o1 = fmaf(w, vx[c].y, o1);
    }
  }
  const float inv = 1.0f / den;
  return pack2h(o0 * inv, o1 * inv);
}

// The QKV projection's split sums and what turns them into queries, keys and values (kernel-side AttnAppend).
__device__ __forceinline__ void hold(HeadPairLoads& ld) {
#pragma unroll
  for (int sp = 0; sp < kHeadPairMaxS; ++sp) asm volatile("" : "+v"(ld.a[sp][0]), "+v"(ld.a[sp][1]));
}

static_assert(kAttnAppendMaxSplits == kHeadPairMaxS, "the launcher's limit is the one of the loads");
struct AppendArgs {
  const float* qkv_part;
  int S;  // <= kHeadPairMaxS
  size_t split_stride;
  const void* q_gain;
  const void* k_gain;
  const float2* rope;
  float eps;
};

// grid: x = kv head, y = row, then set of rows (y >= n_rows), z = split.  block = four waves.
// Row block: the row's segments from skip_segs[row] (or 0) on, up to kLdsSegs per block.  Set block: up to four of
// the leading shared[y - n_rows].n_segs segments for all rows of the set.
// APPEND: q is not read; every block forms the queries of its columns from the split sums, and the last wave of the
// row block that holds a row's last segment forms the row's new key and value, uses them in its last step and then
// writes them into their page.  The pools are therefore not declared read-only in that variant.
// KV8: the pages hold fp8 keys and values (widened to bf16 in registers; scores, softmax and products as for bf16 pages).
// Its step buffers are half as large, and with the q operand in LDS the variant fits three blocks per compute unit.
template <bool APPEND, bool KV8>
__global__ __launch_bounds__(256, KV8 ? 3 : 2) void attn_decode_bf16_kernel(const float* __restrict__ q, const RowMeta* __restrict__ rows,
                                                               const int32_t* __restrict__ block_table, int max_blocks,
                                                               typename PoolPtr<APPEND>::type k_pool,
                                                               typename PoolPtr<APPEND>::type v_pool, float* __restrict__ part,
                                                               int max_segs, int n_q, int n_kv, float scale,
                                                               uint16_t* __restrict__ o_out, int lds_part_offset,
                                                               int lds_q_offset, int n_rows, const int32_t* __restrict__ skip_segs,
                                                               const AttnShared* __restrict__ shared, AppendArgs ap, int spb) {
  extern __shared__ int32_t pages[];  // block-table slice of this row: ceil(ctx/16) entries (+1 pad), then partials
  const int hk = blockIdx.x;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int group = n_q / n_kv;  // <= 8
  const int j = lane & 15, g = lane >> 4;
  const bool is_set = (int)blockIdx.y >= n_rows;  // block-uniform
  // column c of the matrix operand: member c / group of the set (the row itself in a row block), head c % group.
  // Lane (j, g) holds column j and, in a set of more than 16 columns, column j + 16 of a second operand as well.
  int r, n_members = 1, skip = 0, shared_segs = 0;
  int col_row[2];
  if (is_set) {
    const AttnShared* sh = shared + (blockIdx.y - n_rows);
    n_members = sh->n_rows;
    shared_segs = sh->n_segs;
    r = sh->rows[0];
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      const int mj = (j + 16 * c) / group;
      col_row[c] = sh->rows[mj < n_members ? mj : 0];
    }
  } else {
    r = blockIdx.y;
    col_row[0] = col_row[1] = r;
    if (skip_segs) skip = skip_segs[r];
  }
  const int n_cols = n_members * group;   // <= 32 (fp8 pages: <= 16)
  const bool wide = !KV8 && n_cols > 16;  // block-uniform: the set fills a second group of 16 columns
  const bool col_valid[2] = {j < n_cols, j + 16 < n_cols};
  const int col_head[2] = {hk * group + j % group, hk * group + (j + 16) % group};
  const RowMeta rm = rows[r];
  const int ctx = rm.pos + 1;  // keys 0..pos; the row's own key is in its page already, or (APPEND) formed here
  // A set's members may stand at different positions of one 32-key window (rows of one sequence): same steps and
  // segments, and each column is masked at its own length.  r is the member with the longest context.
  const int ctx_col[2] = {is_set ? rows[col_row[0]].pos + 1 : ctx, is_set ? rows[col_row[1]].pos + 1 : ctx};
  const int n_seg = attn_num_segments(ctx);
  const bool in_lds = !is_set && skip == 0 && n_seg <= kLdsSegs;  // merged by this block
  // this block's segments [lo, hi)
  int lo, hi;
  if (is_set) {
    lo = blockIdx.z * 4;
    hi = min(lo + 4, shared_segs);
  } else {
    if ((int)blockIdx.z >= attn_num_splits(n_seg, spb)) return;  // block-uniform
    const int per = n_seg <= kLdsSegs ? kLdsSegs : spb;
    lo = max((int)blockIdx.z * per, skip);
    hi = min((int)blockIdx.z * per + per, n_seg);
  }
  if (lo >= hi) return;  // block-uniform: nothing left for this block
  const int n_blk = (ctx + 15) >> 4;
  const int n_it = (ctx + 31) >> 5;  // 32-key steps
  auto seg_begin = [&](int sgm) { return attn_seg_begin(sgm, n_it, n_seg); };
  int seg = lo + (wave * (hi - lo)) / 4;  // contiguous, balanced share of the block's segments
  const int seg_end = lo + ((wave + 1) * (hi - lo)) / 4;
  const int it_begin = seg_begin(seg), it_end = seg_begin(seg_end);
  const u32x4_t* kb = k_pool + (size_t)hk * kPairU4(KV8);
  const u32x4_t* vb = v_pool + (size_t)hk * kPairU4(KV8);
  if (!APPEND) {
    for (int i = threadIdx.x; i <= n_blk; i += 256)  // entry n_blk duplicates the last page (odd page counts)
      pages[i] = block_table[(size_t)rm.seq * max_blocks + (i < n_blk ? i : n_blk - 1)];
  }

  // ---- APPEND: queries of this block's columns into LDS, the row's new key and value for the appending wave ----
  bool appends = false;  // wave-uniform: this wave owns the row's last step and with it the new key and value
  float* const lds_part = (float*)(pages + lds_part_offset);
  float* const lds_q = (float*)(pages + lds_q_offset);  // [16 columns][128], APPEND only
  // A set block keeps no partials in LDS; in a wide one that area holds the queries of columns 16.. ([16][128],
  // APPEND only) and behind them the q operands of both column groups ([group][hi | lo][matrix-core step][lane]):
  // with two accumulators per lane there are no registers left for them.
  float* const lds_q1 = lds_part;
  u32x4_t* const lds_qopw = (u32x4_t*)(lds_part + 16 * kD);
  uint16_t* const lds_new = (uint16_t*)(lds_q + 16 * kD);  // the row's new key [128] and value [128] as bf16, APPEND only
  // KV8: the q operand lives in LDS ([hi | lo][matrix-core step][lane], 8 KiB) instead of 32 registers per lane, which
  // lets three blocks share a compute unit.  It takes the place of the fp32 queries once those have been read.
  u32x4_t* const lds_qop = (u32x4_t*)lds_q;
  if (APPEND) {
    // Tasks of a wave: the query heads of columns w, w+4, ...; the last wave of the row block that holds the
    // row's last segment also takes the new key and value.  That wave is the only reader of the page entries they
    // belong to (the block's last 32-key step): it puts them into the operands of that step from LDS, and writes
    // them to the page after its last step, when nothing waits for the stores any more.
    // All loads (split sums, rotation, gains, block table) are issued before anything is consumed.
    int set_rows[8] = {0, 0, 0, 0, 0, 0, 0, 0};  // fetched together, ahead of the loads that need them
    if (is_set) {
      const AttnShared* sh = shared + (blockIdx.y - n_rows);
#pragma unroll
      for (int e = 0; e < 8; ++e) set_rows[e] = sh->rows[e];
    }
    auto member_row = [&](int m) {  // m is the same for the whole wave
      const int a = m & 1 ? set_rows[1] : set_rows[0], b = m & 1 ? set_rows[3] : set_rows[2];
      const int c = m & 1 ? set_rows[5] : set_rows[4], d = m & 1 ? set_rows[7] : set_rows[6];
      return m & 4 ? (m & 2 ? d : c) : (m & 2 ? b : a);
    };
    const int uw = __builtin_amdgcn_readfirstlane(wave);  // lets the compiler see that the task choice is per wave
    appends = !is_set && hi == n_seg && uw == 3;
    const int n_tot = (n_q + 2 * n_kv) * kD;
    float2 cs = ap.rope[(size_t)rm.pos * (kD / 2) + lane];  // the rows of a set have one position
    uint32_t gq0 = 0, gq1 = 0, gk0 = 0, gk1 = 0;            // gains as stored (bf16)
    if (ap.q_gain) { gq0 = ((const uint16_t*)ap.q_gain)[lane]; gq1 = ((const uint16_t*)ap.q_gain)[lane + kD / 2]; }
    HeadPairLoads lq[4] = {}, lk = {}, lv = {};  // slots without a task stay zero
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int t = uw + 4 * u;
      if (t < n_cols) {
        const int m = t / group;  // member of the set
        const int trow = is_set ? member_row(m) : r;
        head_pair_issue(lq[u], ap.qkv_part + (size_t)trow * n_tot + (size_t)(hk * group + t % group) * kD, ap.S, ap.split_stride,
                        kD, lane);
      }
    }
    if (appends) {
      const float* row_part = ap.qkv_part + (size_t)r * n_tot;
      head_pair_issue(lk, row_part + (size_t)(n_q + hk) * kD, ap.S, ap.split_stride, kD, lane);
      head_pair_issue(lv, row_part + (size_t)(n_q + n_kv + hk) * kD, ap.S, ap.split_stride, kD, lane);
      if (ap.k_gain) { gk0 = ((const uint16_t*)ap.k_gain)[lane]; gk1 = ((const uint16_t*)ap.k_gain)[lane + kD / 2]; }
    }
    for (int i = threadIdx.x; i <= n_blk; i += 256)  // entry n_blk duplicates the last page (odd page counts)
      pages[i] = block_table[(size_t)rm.seq * max_blocks + (i < n_blk ? i : n_blk - 1)];
    // Everything loaded above is first touched below this line: the empty statements keep the compiler from moving
    // the arithmetic (and with it the waits) up between the loads.
    asm volatile("" : "+v"(cs.x), "+v"(cs.y), "+v"(gq0), "+v"(gq1), "+v"(gk0), "+v"(gk1));
    // Five heads side by side: the (up to) four query columns of this wave and the new key.  Slots without a task
    // carry zeros through the same arithmetic; their results are not stored.
    HeadPair hp[5];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      hold(lq[u]);
      hp[u].cs = cs; hp[u].g0 = bf2f(gq0); hp[u].g1 = bf2f(gq1);
      head_pair_sum(hp[u], lq[u], ap.S);
    }
    hold(lk);
    hold(lv);
    hp[4].cs = cs; hp[4].g0 = bf2f(gk0); hp[4].g1 = bf2f(gk1);
    head_pair_sum(hp[4], lk, ap.S);
    const bool normalise = ap.q_gain != nullptr;
    if (n_cols > 4) {  // block-uniform: several columns per wave
      head_pairs_finish<5>(hp, kD, normalise, ap.eps);
    } else if (appends) {  // wave-uniform: one column and the key
      HeadPair two[2] = {hp[0], hp[4]};
      head_pairs_finish<2>(two, kD, normalise, ap.eps);
      hp[0] = two[0];
      hp[4] = two[1];
    } else {
      HeadPair one[1] = {hp[0]};
      head_pairs_finish<1>(one, kD, normalise, ap.eps);
      hp[0] = one[0];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int t = uw + 4 * u;
      if (t < n_cols) {
        lds_q[t * kD + lane] = hp[u].v0;
        lds_q[t * kD + kD / 2 + lane] = hp[u].v1;
      }
    }
    if (appends) {  // the new key and value, rounded, wait in LDS for this wave's last step
      HeadPair hv;
      head_pair_sum(hv, lv, ap.S);
      if (KV8) {  // as the bytes the page will hold: key [128], then value [128]
        uint8_t* n8 = (uint8_t*)lds_new;
        n8[lane] = (uint8_t)f2fp8(hp[4].v0);
        n8[lane + kD / 2] = (uint8_t)f2fp8(hp[4].v1);
        n8[kD + lane] = (uint8_t)f2fp8(hv.v0);
        n8[kD + lane + kD / 2] = (uint8_t)f2fp8(hv.v1);
      } else {
        lds_new[lane] = (uint16_t)f2bf(hp[4].v0);
        lds_new[lane + kD / 2] = (uint16_t)f2bf(hp[4].v1);
        lds_new[kD + lane] = (uint16_t)f2bf(hv.v0);
        lds_new[kD + lane + kD / 2] = (uint16_t)f2bf(hv.v1);
      }
    }
    if (wide) {  // block-uniform: the same for the columns 16.. of a wide set, in the same arithmetic
      HeadPairLoads lw[4] = {};
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int t = 16 + uw + 4 * u;
        if (t < n_cols)
          head_pair_issue(lw[u], ap.qkv_part + (size_t)member_row(t / group) * n_tot + (size_t)(hk * group + t % group) * kD, ap.S,
                          ap.split_stride, kD, lane);
      }
      HeadPair hw[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        hold(lw[u]);
        hw[u].cs = cs; hw[u].g0 = bf2f(gq0); hw[u].g1 = bf2f(gq1);
        head_pair_sum(hw[u], lw[u], ap.S);
      }
      head_pairs_finish<4>(hw, kD, normalise, ap.eps);
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int t = uw + 4 * u;  // column 16 + t
        if (16 + t < n_cols) {
          lds_q1[t * kD + lane] = hw[u].v0;
          lds_q1[t * kD + kD / 2 + lane] = hw[u].v1;
        }
      }
    }
    __syncthreads();  // pages[] and the queries are in LDS
  }

  // ---- q operand: hi/lo bf16 split; columns beyond the set are zero -------------------------------
  // matrix-core step s of the column whose query is qh: the dims held by lane group g, as the K operand of the page
  // layout has them
  auto split_q = [&](const float* qh, bool valid, int s, u32x4_t& hi, u32x4_t& lo) __attribute__((always_inline)) {
    uint32_t hi16[4], lo16[4];
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
      float x0 = 0.f, x1 = 0.f;
      const int d0 = KV8 ? 64 * (s >> 1) + 16 * g + 8 * (s & 1) + e : 32 * s + 8 * g + e;
      if (valid) { x0 = qh[d0]; x1 = qh[d0 + 1]; }
      const uint32_t h0 = f2bf(x0), h1 = f2bf(x1);
      hi16[e >> 1] = h0 | (h1 << 16);
      lo16[e >> 1] = pack2bf(x0 - bf2f(h0), x1 - bf2f(h1));
    }
    hi = (u32x4_t){hi16[0], hi16[1], hi16[2], hi16[3]};
    lo = (u32x4_t){lo16[0], lo16[1], lo16[2], lo16[3]};
  };
  u32x4_t q_hi[KV8 ? 1 : 4], q_lo[KV8 ? 1 : 4];  // KV8: the step this wave builds for the block
  {
    const float* qh = APPEND ? lds_q + j * kD : q + ((size_t)col_row[0] * n_q + col_head[0]) * kD;
    if constexpr (KV8) {
      split_q(qh, col_valid[0], wave, q_hi[0], q_lo[0]);  // one step per wave, shared through LDS
    } else {
#pragma unroll
      for (int s = 0; s < 4; ++s) split_q(qh, col_valid[0], s, q_hi[s], q_lo[s]);
    }
  }
  if constexpr (KV8) {
    if (APPEND) __syncthreads();  // every wave has read the fp32 queries that the operand overwrites
    lds_qop[wave * 64 + lane] = q_hi[0];
    lds_qop[256 + wave * 64 + lane] = q_lo[0];
  }
  if constexpr (!KV8) {
    if (wide) {  // both groups' operands go through LDS, wave w storing step w
      const float* qh = APPEND ? lds_q1 + j * kD : q + ((size_t)col_row[1] * n_q + col_head[1]) * kD;
      u32x4_t w_hi, w_lo;
      split_q(qh, col_valid[1], wave, w_hi, w_lo);
      const u32x4_t h0 = wave == 0 ? q_hi[0] : wave == 1 ? q_hi[1] : wave == 2 ? q_hi[2] : q_hi[3];
      const u32x4_t l0 = wave == 0 ? q_lo[0] : wave == 1 ? q_lo[1] : wave == 2 ? q_lo[2] : q_lo[3];
      lds_qopw[wave * 64 + lane] = h0;
      lds_qopw[256 + wave * 64 + lane] = l0;
      lds_qopw[512 + wave * 64 + lane] = w_hi;
      lds_qopw[768 + wave * 64 + lane] = w_lo;
    }
  }
  if (!APPEND || KV8 || wide) __syncthreads();  // pages[] is filled; the q operands kept in LDS are complete

  // Segment partials of short contexts (<= kLdsSegs segments) stay in LDS; longer ones and the shared ones go
  // through the workspace.  pcol: this lane's column, indexed by the absolute segment number.
  float* const gcol = part + ((size_t)col_row[0] * n_q + col_head[0]) * max_segs * kPartStride;
  float* const pcol[2] = {in_lds ? lds_part + (size_t)j * n_seg * kPartStride : gcol,
                          part + ((size_t)col_row[1] * n_q + col_head[1]) * max_segs * kPartStride};
  // per column group (the second one only in a wide set)
  f32x4_t o_acc[2][8];
  float m_run[2], l_run[2];
  auto reset = [&](auto ng) __attribute__((always_inline)) {
#pragma unroll
    for (int c = 0; c < decltype(ng)::value; ++c) {
#pragma unroll
      for (int b = 0; b < 8; ++b) o_acc[c][b] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
      m_run[c] = -INFINITY;
      l_run[c] = 0.f;
    }
  };
  reset(std::integral_constant<int, 2>{});
  while (seg < seg_end && seg_begin(seg + 1) == seg_begin(seg)) ++seg;  // skip leading empty segments
  int boundary = seg < seg_end ? seg_begin(seg + 1) : it_end;

  // One step = 32 keys (two pages): scores, online softmax, P*V; at a segment end the partial is written.
  // NG = 2: the same for both column groups of a wide set, from the same key and value registers.
  auto step = [&](const PagePair& pp, int it, auto ng) __attribute__((always_inline)) {
    constexpr int NG = decltype(ng)::value;
    f32x4_t sa[NG], sb[NG];
#pragma unroll
    for (int c = 0; c < NG; ++c) sa[c] = sb[c] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const bool q_in_lds = KV8 || NG == 2;
      const u32x4_t* const qop = KV8 ? lds_qop : lds_qopw;
      const bf16x8_t qa = __builtin_bit_cast(bf16x8_t, q_in_lds ? qop[s * 64 + lane] : q_hi[KV8 ? 0 : s]);
      const bf16x8_t ql = __builtin_bit_cast(bf16x8_t, q_in_lds ? qop[256 + s * 64 + lane] : q_lo[KV8 ? 0 : s]);
      sa[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, pp.k[0][s]), qa, sa[0], 0, 0, 0);
      sa[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, pp.k[0][s]), ql, sa[0], 0, 0, 0);
      sb[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, pp.k[1][s]), qa, sb[0], 0, 0, 0);
      sb[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, pp.k[1][s]), ql, sb[0], 0, 0, 0);
      if constexpr (NG == 2) {
        const bf16x8_t wa = __builtin_bit_cast(bf16x8_t, lds_qopw[512 + s * 64 + lane]);
        const bf16x8_t wl = __builtin_bit_cast(bf16x8_t, lds_qopw[768 + s * 64 + lane]);
        sa[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, pp.k[0][s]), wa, sa[1], 0, 0, 0);
        sa[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, pp.k[0][s]), wl, sa[1], 0, 0, 0);
        sb[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, pp.k[1][s]), wa, sb[1], 0, 0, 0);
        sb[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, pp.k[1][s]), wl, sb[1], 0, 0, 0);
      }
    }
    const int kbase = it * 32 + 4 * g;
    bf16x8_t p_op[NG];
    float alpha[NG];
#pragma unroll
    for (int c = 0; c < NG; ++c) {
      float sc[8];
      float mx = -INFINITY;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        sc[e] = (kbase + e < ctx_col[c]) ? sa[c][e] * scale : -INFINITY;
        sc[4 + e] = (kbase + 16 + e < ctx_col[c]) ? sb[c][e] * scale : -INFINITY;
        mx = fmaxf(mx, fmaxf(sc[e], sc[4 + e]));
      }
      mx = fmaxf(mx, __shfl_xor(mx, 16, kWave));
      mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
      const float m_new = fmaxf(m_run[c], mx);  // finite: key it*32 is inside every column's context
      alpha[c] = __expf(m_run[c] - m_new);
      m_run[c] = m_new;
      uint32_t pw[4];
      float psum = 0.f;
#pragma unroll
      for (int e = 0; e < 8; e += 2) {
        const uint32_t b0 = f2bf(__expf(sc[e] - m_new)), b1 = f2bf(__expf(sc[e + 1] - m_new));
        psum += bf2f(b0) + bf2f(b1);  // the sum uses the rounded weights the product uses
        pw[e >> 1] = b0 | (b1 << 16);
      }
      l_run[c] = l_run[c] * alpha[c] + psum;
      p_op[c] = __builtin_bit_cast(bf16x8_t, (u32x4_t){pw[0], pw[1], pw[2], pw[3]});
    }
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      const int jj = b >> 1, par = b & 1;
      u32x4_t vop;
      vop[0] = pp.v[0][jj][2 * par];
      vop[1] = pp.v[0][jj][2 * par + 1];
      vop[2] = pp.v[1][jj][2 * par];
      vop[3] = pp.v[1][jj][2 * par + 1];
#pragma unroll
      for (int c = 0; c < NG; ++c) {
        o_acc[c][b] *= alpha[c];
        o_acc[c][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, vop), p_op[c], o_acc[c][b], 0, 0, 0);
      }
    }
    if (it + 1 == boundary) {  // wave-uniform
#pragma unroll
      for (int c = 0; c < NG; ++c) {
        float l_tot = l_run[c] + __shfl_xor(l_run[c], 16, kWave);
        l_tot += __shfl_xor(l_tot, 32, kWave);
        if (col_valid[c]) {
          const bool lds_rec = c == 0 && in_lds;  // block-uniform
          float* p = pcol[c] + (lds_rec ? (size_t)seg * kPartStride : part_o(max_segs, seg));
          float* pm = lds_rec ? p + kD : pcol[c] + part_ml(max_segs, seg);
#pragma unroll
          for (int b = 0; b < 8; ++b) {
            p[16 * b + 4 * g] = o_acc[c][b][0]; p[16 * b + 4 * g + 1] = o_acc[c][b][1];
            p[16 * b + 4 * g + 2] = o_acc[c][b][2]; p[16 * b + 4 * g + 3] = o_acc[c][b][3];
          }
          if (g == 0) { pm[0] = m_run[c]; pm[1] = l_tot; }
        }
      }
      // Stores and loads share one counter and may finish out of order, so a store that may be pending makes the
      // compiler turn every later wait for a load into a wait for everything, the other buffer's loads included.
      // Draining the counter here, once per segment, keeps the steps after this branch free of that: they wait
      // only for the loads they consume, and the other buffer stays in flight.
      __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0); expcnt and lgkmcnt at their maxima, i.e. not waited for
      reset(ng);
      ++seg;
      while (seg < seg_end && seg_begin(seg + 1) == seg_begin(seg)) ++seg;
      boundary = seg < seg_end ? seg_begin(seg + 1) : it_end;
    }
  };
  typedef typename std::conditional<KV8, PagePair8, PagePair>::type Buf;  // registers of a step as loaded
  auto fetch = [&](Buf& pp, int it) __attribute__((always_inline)) {
    load_pair(pp, kb, vb, pages[2 * it], pages[2 * it + 1], n_kv, lane);
  };
  auto consume = [&](const Buf& pp, int it, auto ng) __attribute__((always_inline)) {
    if constexpr (KV8) {
      PagePair w;
      widen(w, pp);
      step(w, it, ng);
    } else {
      step(pp, it, ng);
    }
  };

  // The appending wave's last step: the entries of the new token (key pos & 15 of page (pos >> 4) & 1 of the pair)
  // are replaced by the rounded new key and value; what memory holds there is stale.
  auto patch_new = [&](Buf& buf) __attribute__((always_inline)) {
    const int t = rm.pos & 15, pg = (rm.pos >> 4) & 1;
    if constexpr (KV8) {
      const uint8_t* n8 = (const uint8_t*)lds_new;
      // K: the lane whose key is t holds, per load c, the key's dims 64c + 16g .. +15: one 16-byte piece of the new key
      const bool k_lane = (lane & 15) == t;
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        const u32x4_t kn = *(const u32x4_t*)(n8 + 64 * c + 16 * g);
#pragma unroll
        for (int p = 0; p < 2; ++p)
#pragma unroll
          for (int e = 0; e < 4; ++e) buf.k[p][c][e] = (k_lane && pg == p) ? kn[e] : buf.k[p][c][e];
      }
      // V: lanes of key group t >> 2 hold byte t & 3 of word 2*(jj&1) + par = dim 32jj + 16par + dl (dl = lane & 15)
      const bool v_lane = g == (t >> 2);
      const int sh = (t & 3) * 8;
      const uint32_t keep = ~(0xffu << sh);
#pragma unroll
      for (int J = 0; J < 2; ++J)
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const uint32_t vn = (uint32_t)n8[kD + 64 * J + 32 * (w >> 1) + 16 * (w & 1) + j] << sh;
#pragma unroll
          for (int p = 0; p < 2; ++p) {
            const uint32_t old = buf.v[p][J][w];
            buf.v[p][J][w] = (v_lane && pg == p) ? ((old & keep) | vn) : old;
          }
        }
      return;
    } else {
    PagePair& pp = buf;
    // K operand: the lane whose row is key t holds 8 dims per step, one 16-byte piece of the new key
    const bool k_lane = (lane & 15) == t;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const u32x4_t kn = *(const u32x4_t*)(lds_new + 32 * s + 8 * g);
#pragma unroll
      for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int e = 0; e < 4; ++e) pp.k[p][s][e] = (k_lane && pg == p) ? kn[e] : pp.k[p][s][e];
    }
    // V operand: keys 4g..4g+3 of dims 32jj + dl (registers 0, 1) and 32jj + 16 + dl (registers 2, 3)
    const bool v_lane = g == (t >> 2);
    const int sh = (t & 1) * 16, hi_pair = (t >> 1) & 1;
    const uint32_t keep = ~(0xffffu << sh);
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
#pragma unroll
      for (int par = 0; par < 2; ++par) {
        const uint32_t vn = (uint32_t)lds_new[kD + (2 * jj + par) * 16 + j] << sh;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
#pragma unroll
          for (int p = 0; p < 2; ++p) {
            const uint32_t old = pp.v[p][jj][2 * par + h];
            pp.v[p][jj][2 * par + h] = (v_lane && h == hi_pair && pg == p) ? ((old & keep) | vn) : old;
          }
        }
      }
    }
    }
  };
  // ... and its stores, once nothing of the wave's work is behind them
  auto store_new = [&]() __attribute__((always_inline)) {
    const int t = rm.pos & 15;
    if constexpr (KV8) {
      const uint8_t* n8 = (const uint8_t*)lds_new;
      kv_store_fp8_bits((void*)k_pool, rm.page, hk, n_kv, t, lane, n8[lane], false);
      kv_store_fp8_bits((void*)k_pool, rm.page, hk, n_kv, t, lane + kD / 2, n8[lane + kD / 2], false);
      kv_store_fp8_bits((void*)v_pool, rm.page, hk, n_kv, t, lane, n8[kD + lane], true);
      kv_store_fp8_bits((void*)v_pool, rm.page, hk, n_kv, t, lane + kD / 2, n8[kD + lane + kD / 2], true);
      return;
    }
    kv_store_bf16_bits((void*)k_pool, rm.page, hk, n_kv, t, lane, lds_new[lane], false);
    kv_store_bf16_bits((void*)k_pool, rm.page, hk, n_kv, t, lane + kD / 2, lds_new[lane + kD / 2], false);
    kv_store_bf16_bits((void*)v_pool, rm.page, hk, n_kv, t, lane, lds_new[kD + lane], true);
    kv_store_bf16_bits((void*)v_pool, rm.page, hk, n_kv, t, lane + kD / 2, lds_new[kD + lane + kD / 2], true);
  };

  // Two register buffers, refilled unconditionally inside the loop so that the compiler's wait counts let the
  // other buffer's 16 loads stay in flight while one is consumed; the ragged end is peeled off below.
  auto run = [&](auto ng) __attribute__((always_inline)) {
    constexpr bool kRow = decltype(ng)::value == 1;  // only a row block appends
    if (it_begin < it_end) {
      Buf pa, pb;
      fetch(pa, it_begin);
      int it = it_begin;
      for (; it + 2 < it_end; it += 2) {
        fetch(pb, it + 1);
        __builtin_amdgcn_sched_barrier(0);
        consume(pa, it, ng);
        __builtin_amdgcn_sched_barrier(0);
        fetch(pa, it + 2);
        __builtin_amdgcn_sched_barrier(0);
        consume(pb, it + 1, ng);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (it + 1 < it_end) {  // two steps left
        fetch(pb, it + 1);
        __builtin_amdgcn_sched_barrier(0);
        consume(pa, it, ng);
        if (APPEND && kRow && appends) patch_new(pb);
        consume(pb, it + 1, ng);
      } else {  // one step left
        if (APPEND && kRow && appends) patch_new(pa);
        consume(pa, it, ng);
      }
    }
  };
  if (wide) {
    if constexpr (!KV8) run(std::integral_constant<int, 2>{});
  } else {
    run(std::integral_constant<int, 1>{});
  }

  if (!in_lds) {  // the merge kernel combines the partials in the workspace
    if (APPEND && appends) store_new();
    return;
  }
  // ---- merge: wave w takes heads w, w+4 of the group -------------------------------------------------
  __threadfence_block();
  __syncthreads();
  for (int hh = wave; hh < group; hh += 4) {
    const int head = hk * group + hh;
    const float* p = lds_part + (size_t)hh * n_seg * kPartStride;
    const uint32_t o2 = merge_short([&](int c) { return p + (size_t)c * kPartStride; },
                                    [&](int c) { return p + (size_t)c * kPartStride + kD; }, n_seg, n_it, lane);
    *(uint32_t*)(o_out + frag_offset(r, head * kD + 2 * lane, (n_q * kD) >> 6)) = o2;
  }
  if (APPEND && appends) store_new();
}

// Merge of the rows whose partials are in the workspace, one wave per (row, head): rows of a set (short contexts:
// the arithmetic of the in-block merge) and long-context rows (more than kLdsSegs segments, none of them empty).
// For the latter the segment weights exp(m_c - M) are formed by the lanes in parallel (max and denominator by the wave's fixed
// butterfly), then the O partials are accumulated in index order, eight loads in flight at a time.  Rows with
// short contexts were finished by the first kernel.
__global__ __launch_bounds__(64) void attn_merge_bf16_kernel(const float* __restrict__ part, const RowMeta* __restrict__ rows,
                                                             int max_segs, uint16_t* __restrict__ o_out, int n_q,
                                                             const int32_t* __restrict__ skip_segs) {
  const int head = blockIdx.x, r = blockIdx.y, lane = threadIdx.x;
  const int ctx = rows[r].pos + 1;
  const int n_seg = attn_num_segments(ctx);
  const float* p = part + ((size_t)r * n_q + head) * max_segs * kPartStride;
  if (n_seg <= kLdsSegs) {
    if (!skip_segs || skip_segs[r] == 0) return;  // finished by its own block
    const uint32_t o2 = merge_short([&](int c) { return p + part_o(max_segs, c); }, [&](int c) { return p + part_ml(max_segs, c); },
                                    n_seg, (ctx + 31) >> 5, lane);
    *(uint32_t*)(o_out + frag_offset(r, head * kD + 2 * lane, (n_q * kD) >> 6)) = o2;
    return;
  }
  constexpr int kMaxPerLane = 4;  // up to 256 segments = contexts up to 65536
  float mc[kMaxPerLane], lc[kMaxPerLane];
  float M = -INFINITY;
#pragma unroll
  for (int u = 0; u < kMaxPerLane; ++u) {
    const int c = lane + 64 * u;
    mc[u] = -INFINITY;
    lc[u] = 0.f;
    if (c < n_seg) {
      const float2 ml = *(const float2*)(p + part_ml(max_segs, c));
      mc[u] = ml.x;
      lc[u] = ml.y;
    }
    M = fmaxf(M, mc[u]);
  }
  M = wave_max(M);
  float den = 0.f;
#pragma unroll
  for (int u = 0; u < kMaxPerLane; ++u) {
    mc[u] = __expf(mc[u] - M);  // weight of segment lane + 64u (0 beyond n_seg)
    den += mc[u] * lc[u];
  }
  den = wave_sum(den);
  float o0 = 0.f, o1 = 0.f;
#pragma unroll
  for (int u = 0; u < kMaxPerLane; ++u) {
    const int c_end = min(64, n_seg - 64 * u);  // a multiple of 4, like n_seg
    for (int cl = 0; cl < c_end; cl += 4) {
      float2 v[4];
      float w[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        v[e] = *(const float2*)(p + part_o(max_segs, 64 * u + cl + e) + 2 * lane);
        w[e] = __shfl(mc[u], cl + e, kWave);
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        o0 += w[e] * v[e].x;
        o1 += w[e] * v[e].y;
      }
    }
  }
  const float inv = 1.0f / den;
  *(uint32_t*)(o_out + frag_offset(r, head * kD + 2 * lane, (n_q * kD) >> 6)) = pack2h(o0 * inv, o1 * inv);
}

}  // namespace

// Segment records to allocate per (row, head): a multiple of 16, which keeps every O row of the workspace on whole
// cache lines.
int attn_bf16_max_segments(int max_ctx) { return (attn_num_segments(max_ctx) + 15) & ~15; }

bool launch_attn_decode_bf16(hipStream_t s, const Geometry& g, const float* q, const RowMeta* rows,
                             const int32_t* block_table, void* k_pool_layer, void* v_pool_layer, float* part,
                             int max_segs_alloc, int max_ctx_in_batch, void* o_out, int M, const int32_t* skip_segs,
                             const AttnShared* shared, int n_shared, int max_shared_segs, const AttnAppend* append,
                             int segs_per_block) {
  const int n_seg_max = attn_num_segments(max_ctx_in_batch);
  const int spb = std::min(std::max(segs_per_block, 1), kLdsSegs);
  const int page_ints = ((max_ctx_in_batch + 15) / 16 + 1 + 3) & ~3;  // keeps the partials 16-byte aligned
  if (n_shared <= 0) { skip_segs = nullptr; n_shared = 0; max_shared_segs = 0; }
  const int z = std::max(attn_num_splits(n_seg_max, spb), (max_shared_segs + 3) / 4);
  dim3 grid(g.n_kv, M + n_shared, z);
  const int segs = n_seg_max > kLdsSegs ? kLdsSegs : n_seg_max;
  int part_floats = (g.n_q / g.n_kv) * segs * kPartStride;  // a multiple of 4
  // a set of more than 16 columns keeps the queries of its columns 16.. and the two q operands there
  if (n_shared > 0 && !g.kv_fp8) part_floats = std::max(part_floats, 3 * 16 * kD);
  // the queries of up to 16 columns, the new key and value (bf16); fp8 pages: the q operand (in the queries' place)
  const int q_ints = append ? 16 * kD + kD : g.kv_fp8 ? 16 * kD : 0;
  const size_t lds = (size_t)(page_ints + part_floats + q_ints) * 4;
  const float scale = 1.0f / sqrtf((float)g.head_dim);
  AppendArgs ap = {};
  if (append) {
    ap.qkv_part = append->qkv_part; ap.S = append->S;
    ap.split_stride = (size_t)M * (g.n_q + 2 * g.n_kv) * g.head_dim;
    ap.q_gain = append->q_gain; ap.k_gain = append->k_gain; ap.rope = append->rope_table; ap.eps = g.rms_eps;
  }
#define RL_ATTN_LAUNCH(APP, K8)                                                                                          \
  attn_decode_bf16_kernel<APP, K8><<<grid, 256, lds, s>>>(q, rows, block_table, g.max_blocks, (const u32x4_t*)k_pool_layer, \
                                                          (const u32x4_t*)v_pool_layer, part, max_segs_alloc, g.n_q, g.n_kv, \
                                                          scale, (uint16_t*)o_out, page_ints, page_ints + part_floats, M,  \
                                                          skip_segs, shared, ap, spb)
  if (append) {
    if (g.kv_fp8) RL_ATTN_LAUNCH(true, true); else RL_ATTN_LAUNCH(true, false);
  } else {
    if (g.kv_fp8) RL_ATTN_LAUNCH(false, true); else RL_ATTN_LAUNCH(false, false);
  }
#undef RL_ATTN_LAUNCH
  return n_seg_max > kLdsSegs || n_shared > 0;
}

void launch_attn_merge_bf16(hipStream_t s, const Geometry& g, const RowMeta* rows, float* part, int max_segs_alloc,
                            void* o_out, int M, const int32_t* skip_segs, int n_shared) {
  if (n_shared <= 0) skip_segs = nullptr;
  attn_merge_bf16_kernel<<<dim3(g.n_q, M), 64, 0, s>>>(part, rows, max_segs_alloc, (uint16_t*)o_out, g.n_q, skip_segs);
}

}  // namespace rl
