// Stand-alone Gumbel-max sampling kernels (logits in memory) and the merge stage shared with the fused path.
// The arithmetic contract lives in sampler_device.h.  The log-probability log softmax(z/T)[token] is accumulated
// in fp32 (tolerance, not bit-exact).
#include <mutex>

#include "../../include/rl.h"
#include "kernels.h"
#include "sampler_device.h"

namespace rl {

namespace {

// Stage 1: grid (tiles, rows); each block scans kSampleTile vocabulary entries of one row of fp32 logits.
__global__ __launch_bounds__(256) void sample_stage1_kernel(const float* __restrict__ logits, int V,
                                                            const RowMeta* __restrict__ rows, int pos_offset, float inv_t,
                                                            int greedy, uint32_t seed_lo, uint32_t seed_hi,
                                                            const int32_t* __restrict__ forced, float* __restrict__ forced_z,
                                                            float* __restrict__ part, int n_tiles,
                                                            const OrderCut* __restrict__ cuts) {
  __shared__ float sh_y[4], sh_z[4], sh_m[4], sh_s[4];
  __shared__ int sh_i[4];
  const int tile = blockIdx.x, r = blockIdx.y;
  const RowMeta rm = rows[r];
  const uint32_t pos = (uint32_t)(rm.pos + pos_offset), seq = (uint32_t)rm.seq;
  const float* z = logits + (size_t)r * V;
  const int f = forced ? forced[r] : -1;
  OrderCut cut{0u, 0x7fffffff};  // keeps everything
  if (cuts) cut = cuts[r];
  Best best{-INFINITY, -1, 0.f};
  float m = -INFINITY, s = 0.f;
  const int i_end = min(V, (tile + 1) * kSampleTile);
  for (int i0 = tile * kSampleTile + threadIdx.x * 4; i0 < i_end; i0 += 256 * 4) {
    uint32_t rnd[4] = {0, 0, 0, 0};
    if (!greedy) philox4x32_10((uint32_t)i0 >> 2, pos, seq, 0u, seed_lo, seed_hi, rnd);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int i = i0 + e;
      if (i >= i_end) break;
      const float zi = z[i];
      if (!kept_by(cut, order_key(zi), i)) {  // cut off by top-k / top-p: probability zero
        if (i == f) forced_z[r] = -INFINITY;
        continue;
      }
      const float y = greedy ? zi : __fmaf_rn(zi, inv_t, gumbel(rnd[e]));
      best = better(best, Best{y, i, zi});
      lse_merge(m, s, zi * inv_t, 1.0f);
      if (i == f) forced_z[r] = zi;
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    best = better(best, shfl_xor_best(best, o));
    lse_merge(m, s, __shfl_xor(m, o, kWave), __shfl_xor(s, o, kWave));
  }
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { sh_y[wave] = best.y; sh_i[wave] = best.idx; sh_z[wave] = best.z; sh_m[wave] = m; sh_s[wave] = s; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w) {
      best = better(best, Best{sh_y[w], sh_i[w], sh_z[w]});
      lse_merge(m, s, sh_m[w], sh_s[w]);
    }
    float* p = part + ((size_t)r * n_tiles + tile) * kSamplePartFloats;
    *(float4*)p = make_float4(best.y, __int_as_float(best.idx), best.z, 0.f);
    *(float4*)(p + 4) = make_float4(m, s, 0.f, 0.f);
  }
}

// Stage 2: one block of 1024 threads per row merges the tile partials and emits token and log-probability.
__global__ __launch_bounds__(1024) void sample_stage2_kernel(const float* __restrict__ part, int n_tiles, int V,
                                                             const int32_t* __restrict__ forced,
                                                             const float* __restrict__ forced_z, float inv_t,
                                                             int32_t* __restrict__ out_tok, float* __restrict__ out_lp,
                                                             const RowMeta* __restrict__ rows, int32_t* __restrict__ last_tok) {
  __shared__ float sh_y[16], sh_z[16], sh_m[16], sh_s[16];
  __shared__ int sh_i[16];
  const int r = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  Best best{-INFINITY, -1, 0.f};
  float m = -INFINITY, s = 0.f;
  for (int t = threadIdx.x; t < n_tiles; t += 1024) {
    const float* p = part + ((size_t)r * n_tiles + t) * kSamplePartFloats;
    const float4 a = *(const float4*)p;
    const float4 b = *(const float4*)(p + 4);
    best = better(best, Best{a.x, __float_as_int(a.y), a.z});
    lse_merge(m, s, b.x, b.y);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    best = better(best, shfl_xor_best(best, o));
    lse_merge(m, s, __shfl_xor(m, o, kWave), __shfl_xor(s, o, kWave));
  }
  if (lane == 0) { sh_y[wave] = best.y; sh_i[wave] = best.idx; sh_z[wave] = best.z; sh_m[wave] = m; sh_s[wave] = s; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 16; ++w) {
      best = better(best, Best{sh_y[w], sh_i[w], sh_z[w]});
      lse_merge(m, s, sh_m[w], sh_s[w]);
    }
    int tok = best.idx < 0 ? 0 : best.idx;  // idx < 0 only when every score was NaN
    float zt = best.z;
    if (forced != nullptr && forced[r] >= 0 && forced[r] < V) { tok = forced[r]; zt = forced_z[r]; }
    out_tok[r] = tok;
    if (last_tok != nullptr) last_tok[rows[r].seq] = tok;  // what the sequence is fed next when the caller passes no tokens
    out_lp[r] = zt * inv_t - (m + logf(s));
  }
}


// ------------------------------------------------------------------------------------------------
// Top-k / top-p cut of every row: the last kept token of the order, found by radix selection.  A selection runs in
// five stages, three over the digits of the order key from the top (11, 11, 10 bits; count or integer mass per bin,
// bins scanned from the largest down until the target is reached) and two over the digits of the index (11, 11 bits,
// ascending) among the tokens that share the cut's key.  Each stage is one launch with several blocks per row: a
// block first redoes the scan of the previous stage's histogram (every block gets the same answer), then adds its
// slice of the row to this stage's histogram in LDS and from there to the row's histogram in memory.  Integer masses
// make every sum exact, whatever its order, so the cut is reproducible bit for bit.
// ------------------------------------------------------------------------------------------------
constexpr int kCutBins = 2048;
constexpr int kCutStages = 5;

struct CutState {  // after the scan of a stage's histogram
  uint32_t prefix;   // selected digits of the order key so far
  uint32_t iprefix;  // selected digits of the index so far
  unsigned long long rem;  // count or mass still to be covered inside the selection
};
struct CutRow {  // per row, zeroed before a selection starts
  unsigned long long hist[2 * kCutStages][kCutBins];
  CutState st[2 * kCutStages];
  uint32_t kmax;
  uint32_t pad;
};

__device__ __forceinline__ int cut_shift(int stage) { return stage == 0 ? 21 : stage == 1 ? 10 : stage == 2 ? 0 : stage == 3 ? 11 : 0; }
__device__ __forceinline__ int cut_width(int stage) { return stage == 2 ? 10 : 11; }

// Calls fn(i, z[i]) for the tokens of float4 groups [g_begin, g_end) of the row (V % 4 == 0, rows 16-byte aligned),
// eight 16-byte loads in flight per thread.
template <typename F>
__device__ __forceinline__ void for_each_token(const float* __restrict__ z, int g_begin, int g_end, int tid, int nthr, F fn) {
  for (int g0 = g_begin + tid; g0 < g_end; g0 += 8 * nthr) {
    float4 v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int g = g0 + e * nthr;
      v[e] = g < g_end ? ((const float4*)z)[g] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int g = g0 + e * nthr;
      if (g < g_end) { fn(4 * g, v[e].x); fn(4 * g + 1, v[e].y); fn(4 * g + 2, v[e].z); fn(4 * g + 3, v[e].w); }
    }
  }
}

// One wave: the position (in scan order: descending or ascending bin) at which the running sum of `hist` first
// reaches `rem`; the last position is taken when none does.  Returns the bin; *rem_out = what is still to be covered
// inside it; *total_out = sum of all bins.  Every lane returns the same values.
template <bool kDescending, int kPer>
__device__ __forceinline__ int scan_select_n(const unsigned long long* __restrict__ hist, unsigned long long rem, int lane,
                                             unsigned long long* rem_out) {
  constexpr int n_bins = 64 * kPer;
  // this lane's kPer positions (consecutive in scan order), loaded once as 16-byte pairs
  unsigned long long c[kPer];
  const int first = kDescending ? n_bins - (lane + 1) * kPer : lane * kPer;  // lowest bin of the lane's range
#pragma unroll
  for (int e = 0; e < kPer; e += 2) {
    const ulonglong2 v = *(const ulonglong2*)(hist + first + e);
    c[kDescending ? kPer - 1 - e : e] = v.x;
    c[kDescending ? kPer - 2 - e : e + 1] = v.y;
  }
  unsigned long long local = 0;
#pragma unroll
  for (int e = 0; e < kPer; ++e) local += c[e];
  unsigned long long incl = local;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const unsigned long long t = __shfl_up(incl, o, kWave);
    if (lane >= o) incl += t;
  }
  unsigned long long cum = incl - local;  // sum of the positions before this lane's
  int hit = -1;
  unsigned long long before = 0;
#pragma unroll
  for (int e = 0; e < kPer; ++e) {
    const int pos = lane * kPer + e;
    if (hit < 0 && pos < n_bins - 1 && cum + c[e] >= rem) { hit = pos; before = cum; }
    if (pos < n_bins - 1) cum += c[e];  // in the last lane: ends as the sum of all positions but the last
  }
  const unsigned long long any = __ballot(hit >= 0);
  const int src = any ? (int)__builtin_ctzll(any) : 63;
  if (!any) { hit = n_bins - 1; before = cum; }
  hit = __shfl(hit, src, kWave);
  before = __shfl(before, src, kWave);
  *rem_out = rem - before;
  return kDescending ? n_bins - 1 - hit : hit;
}
template <bool kDescending>
__device__ __forceinline__ int scan_select(const unsigned long long* __restrict__ hist, int n_bins, unsigned long long rem,
                                           int lane, unsigned long long* rem_out) {
  return n_bins == 2048 ? scan_select_n<kDescending, 32>(hist, rem, lane, rem_out)
                        : scan_select_n<kDescending, 16>(hist, rem, lane, rem_out);
}

__device__ __forceinline__ unsigned long long wave_total(const unsigned long long* __restrict__ hist, int n_bins, int lane) {
  unsigned long long s = 0;
  for (int b = lane; b < n_bins; b += 64) s += hist[b];
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, kWave);
  return s;
}

// Four (bin, count-or-mass) entries in registers.  The top digit of the order key takes only a handful of values over
// a row of logits, so in the first stage nearly every token would hit the same few LDS words; a thread collects them
// here and adds each entry to the histogram once.
struct BinCache {
  int bin[4];
  unsigned long long val[4];
  int next;
  __device__ __forceinline__ void init() {
#pragma unroll
    for (int e = 0; e < 4; ++e) { bin[e] = -1; val[e] = 0; }
    next = 0;
  }
  __device__ __forceinline__ void add(int b, unsigned long long w, unsigned long long* h) {
    bool hit = false;
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (bin[e] == b) { val[e] += w; hit = true; }
    if (hit) return;
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (next == e) {
        if (bin[e] >= 0) atomicAdd(&h[bin[e]], val[e]);
        bin[e] = b;
        val[e] = w;
      }
    next = (next + 1) & 3;
  }
  __device__ __forceinline__ void flush(unsigned long long* h) {
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (bin[e] >= 0) atomicAdd(&h[bin[e]], val[e]);
  }
};

__global__ __launch_bounds__(256) void cut_zero_kernel(CutRow* __restrict__ ws) {
  uint4* p = (uint4*)(ws + blockIdx.y);
  const int n = (int)(sizeof(CutRow) / 16);
  for (int i = blockIdx.x * 256 + threadIdx.x; i < n; i += gridDim.x * 256) p[i] = make_uint4(0u, 0u, 0u, 0u);
}

// grid (slices, rows): largest order key of the row -> ws[row].kmax
__global__ __launch_bounds__(256) void cut_kmax_kernel(const float* __restrict__ logits, int V, CutRow* __restrict__ ws) {
  const int r = blockIdx.y, tid = threadIdx.x;
  const float* z = logits + (size_t)r * V;
  const int n4 = V >> 2, per = (n4 + gridDim.x - 1) / gridDim.x;
  const int g_begin = blockIdx.x * per, g_end = min(n4, g_begin + per);
  uint32_t kmax = 0;
  for_each_token(z, g_begin, g_end, tid, 256, [&](int, float zi) { kmax = max(kmax, order_key(zi)); });
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, o, kWave));
  if ((tid & 63) == 0 && kmax != 0) atomicMax(&ws[r].kmax, kmax);
}

// Stage `stage` (0..4) of selection `sel` (0: first, 1: second) of every row; stage == kCutStages only finishes the
// selection and writes the cut.  kMass: bins hold integer masses and the first stage's target is
// max(1, floor(p_fixed * S / 2^32)), S = mass of all allowed tokens (p_fixed == 0: the target is `target`);
// otherwise bins hold counts and the target is `target`.  allowed_cuts (may be null): only tokens kept by that
// earlier cut take part.
template <bool kMass>
__global__ __launch_bounds__(256) void cut_stage_kernel(const float* __restrict__ logits, int V, float inv_t, int stage, int sel,
                                                        unsigned long long target, unsigned long long p_fixed,
                                                        const OrderCut* __restrict__ allowed_cuts,
                                                        CutRow* __restrict__ ws, OrderCut* __restrict__ cuts_out) {
  __shared__ unsigned long long lh[kCutBins];
  __shared__ CutState sh_st;
  const int r = blockIdx.y, tid = threadIdx.x, lane = tid & 63;
  CutRow& row = ws[r];
  const int slot = sel * kCutStages + stage;
  const float* z = logits + (size_t)r * V;
  const float s_max = __fmul_rn(order_value(row.kmax), inv_t);
  OrderCut allowed{0u, 0x7fffffff};
  if (allowed_cuts) allowed = allowed_cuts[r];

  // ---- state after the previous stage (first wave; the answer is the same in every block of the row) ----------
  if (tid < 64) {
    CutState st{0u, 0u, target};
    if (stage > 0) {
      const unsigned long long* ph = row.hist[slot - 1];
      const int pbins = 1 << cut_width(stage - 1);
      if (stage == 1) {
        if (kMass && p_fixed != 0) {
          const unsigned long long S = wave_total(ph, pbins, lane);
          st.rem = (__umul64hi(S, p_fixed) << 32) | ((S * p_fixed) >> 32);  // S < 2^50, p_fixed < 2^32
          if (st.rem < 1) st.rem = 1;
        }
      } else {
        st = row.st[slot - 2];
      }
      unsigned long long rem_out;
      if (stage <= 3) {  // previous stage was a key digit: scan from the largest bin down
        const int b = scan_select<true>(ph, pbins, st.rem, lane, &rem_out);
        st.prefix |= (uint32_t)b << cut_shift(stage - 1);
        if (stage == 3) {  // key complete: tokens with this key, in ascending index order -- how many are needed
          if (kMass) {
            const unsigned long long w = fexp_weight(__fmaf_rn(order_value(st.prefix), inv_t, -s_max));
            rem_out = w > 0 ? (rem_out + w - 1) / w : 1ull;
          }
          if (rem_out < 1) rem_out = 1;
        }
      } else {           // previous stage was an index digit: scan upwards
        const int b = scan_select<false>(ph, pbins, st.rem, lane, &rem_out);
        st.iprefix |= (uint32_t)b << cut_shift(stage - 1);
      }
      st.rem = rem_out;
      if (blockIdx.x == 0 && lane == 0) {
        if (stage < kCutStages) row.st[slot - 1] = st;
        else cuts_out[r] = OrderCut{st.prefix, (int32_t)st.iprefix};
      }
    }
    if (lane == 0) sh_st = st;
  }
  if (stage == kCutStages) return;  // block-uniform
  for (int b = tid; b < kCutBins; b += 256) lh[b] = 0ull;
  __syncthreads();
  const CutState st = sh_st;

  // ---- this block's slice of the row into the stage's histogram ------------------------------------------
  const int n4 = V >> 2, per = (n4 + gridDim.x - 1) / gridDim.x;
  const int g_begin = blockIdx.x * per, g_end = min(n4, g_begin + per);
  const int shift = cut_shift(stage), mask = (1 << cut_width(stage)) - 1;
  if (stage == 0) {
    BinCache bc;
    bc.init();
    for_each_token(z, g_begin, g_end, tid, 256, [&](int i, float zi) {
      const uint32_t k = order_key(zi);
      if (!kept_by(allowed, k, i)) return;
      bc.add((int)(k >> shift), kMass ? fexp_weight(__fmaf_rn(zi, inv_t, -s_max)) : 1ull, lh);
    });
    bc.flush(lh);
  } else if (stage < 3) {
    const int above = shift + cut_width(stage);
    for_each_token(z, g_begin, g_end, tid, 256, [&](int i, float zi) {
      const uint32_t k = order_key(zi);
      if ((k >> above) != (st.prefix >> above) || !kept_by(allowed, k, i)) return;
      atomicAdd(&lh[(k >> shift) & mask], kMass ? fexp_weight(__fmaf_rn(zi, inv_t, -s_max)) : 1ull);
    });
  } else {
    for_each_token(z, g_begin, g_end, tid, 256, [&](int i, float zi) {
      const uint32_t k = order_key(zi);
      if (k != st.prefix || !kept_by(allowed, k, i)) return;
      if (stage == 4 && ((uint32_t)i >> 11) != (st.iprefix >> 11)) return;
      atomicAdd(&lh[((uint32_t)i >> shift) & mask], 1ull);
    });
  }
  __syncthreads();
  for (int b = tid; b < kCutBins; b += 256)
    if (lh[b] != 0ull) atomicAdd(&row.hist[slot][b], lh[b]);
}

}  // namespace

size_t sample_cut_bytes_per_row() { return sizeof(CutRow) + 2 * sizeof(OrderCut); }

void launch_sample(hipStream_t st, const float* logits, int M, int V, const RowMeta* rows, int pos_offset,
                   const int32_t* forced, float temperature, uint64_t seed, float* part, float* forced_z,
                   int32_t* out_tokens, float* out_logprobs, int top_k, float top_p, void* cut_buf, int32_t* last_tok) {
  const int n_tiles = (V + kSampleTile - 1) / kSampleTile;
  const int greedy = !(temperature > 0.f);
  const float inv_t = greedy ? 1.0f : 1.0f / temperature;
  dim3 grid(n_tiles, M);
  const OrderCut* cuts = nullptr;
  if (!greedy && sample_is_truncated(V, top_k, top_p)) {  // greedy ignores the cuts: the argmax is always kept
    CutRow* ws = (CutRow*)cut_buf;
    OrderCut* cut_k = (OrderCut*)((char*)cut_buf + (size_t)M * sizeof(CutRow));  // [M] after top-k, then [M] final
    OrderCut* cut_p = cut_k + M;
    int slices = 512 / M;
    slices = slices < 1 ? 1 : (slices > 64 ? 64 : slices);
    const dim3 sg(slices, M);
    cut_zero_kernel<<<dim3(8, M), 256, 0, st>>>(ws);
    cut_kmax_kernel<<<sg, 256, 0, st>>>(logits, V, ws);
    const bool use_k = top_k > 0 && top_k < V, use_p = top_p > 0.0f && top_p < 1.0f;
    const OrderCut* allowed = nullptr;
    if (use_k) {
      for (int stage = 0; stage <= kCutStages; ++stage)
        cut_stage_kernel<false><<<stage < kCutStages ? sg : dim3(1, M), 256, 0, st>>>(logits, V, inv_t, stage, 0,
                                                                                    (unsigned long long)top_k, 0ull, nullptr, ws, cut_k);
      allowed = cut_k;
      cuts = cut_k;
    }
    if (use_p) {
      const unsigned long long P = (unsigned long long)(top_p * 4294967296.0f);  // exact scaling, truncated
      for (int stage = 0; stage <= kCutStages; ++stage)
        cut_stage_kernel<true><<<stage < kCutStages ? sg : dim3(1, M), 256, 0, st>>>(logits, V, inv_t, stage, 1, 1ull, P, allowed,
                                                                                   ws, cut_p);
      cuts = cut_p;
    }
  }
  sample_stage1_kernel<<<grid, 256, 0, st>>>(logits, V, rows, pos_offset, inv_t, greedy, (uint32_t)(seed & 0xffffffffu),
                                             (uint32_t)(seed >> 32), forced, forced_z, part, n_tiles, cuts);
  sample_stage2_kernel<<<M, 1024, 0, st>>>(part, n_tiles, V, forced, forced_z, inv_t, out_tokens, out_logprobs, rows, last_tok);
}

void launch_sample_merge(hipStream_t st, const float* part, int n_tiles, int M, int V, const int32_t* forced,
                         const float* forced_z, float temperature, int32_t* out_tokens, float* out_logprobs,
                         const RowMeta* rows, int32_t* last_tok) {
  const float inv_t = temperature > 0.f ? 1.0f / temperature : 1.0f;
  sample_stage2_kernel<<<M, 1024, 0, st>>>(part, n_tiles, V, forced, forced_z, inv_t, out_tokens, out_logprobs, rows, last_tok);
}

}  // namespace rl

// ------------------------------------------------------------------------------------------------
// The plain sampler for callers that cannot allocate (code under graph capture, serving loops, harnesses that forbid
// it): the same two kernels as above, with the row metadata, the forced tokens' logits and the per-tile partials in
// a file-scope device array instead of a model's workspace.  Each GPU has its own copy of the array at its own
// address; that address is looked up once per device and used from then on (the array's name is not a device
// address in host code).  Every call on a GPU uses that GPU's array, so calls that overlap on one GPU race.
// ------------------------------------------------------------------------------------------------
namespace rl {

namespace {

constexpr int kStaticRows = 256;          // rows per call
constexpr int kStaticTileRows = 20480;    // rows x ceil(vocab / kSampleTile) per call (151 936 entries x 256 rows: 19 200)
constexpr size_t kStaticRowsOff = 0;                                           // RowMeta [kStaticRows]
constexpr size_t kStaticForcedOff = kStaticRowsOff + kStaticRows * sizeof(RowMeta);  // float [kStaticRows]
constexpr size_t kStaticPartOff = kStaticForcedOff + kStaticRows * sizeof(float);    // float [kStaticTileRows][8]
constexpr size_t kStaticBytes = kStaticPartOff + (size_t)kStaticTileRows * kSamplePartFloats * sizeof(float);
static_assert(kStaticPartOff % 16 == 0, "the partials are written as float4");

static __device__ __align__(256) unsigned char scratch[kStaticBytes];  // 660 480 bytes per GPU, held until the process ends

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
unsigned char* g_scratch_ptr[kMaxDevices] = {};

// Address of the current device's copy of `scratch` (looked up on first use on that device).
hipError_t scratch_address(unsigned char** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    g_scratch_ptr[dev] = (unsigned char*)p;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

__global__ __launch_bounds__(256) void static_rows_kernel(const int32_t* __restrict__ seq_ids, const int32_t* __restrict__ positions,
                                                          RowMeta* __restrict__ rows, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) rows[i] = RowMeta{seq_ids[i], positions[i], 0, 0};
}

}  // namespace

}  // namespace rl

extern "C" rl_status rl_sample_logits_static(void* stream, int32_t n, int32_t vocab, const float* logits,
                                             const int32_t* seq_ids, const int32_t* positions, const int32_t* forced,
                                             const rl_sampling* sp, int32_t* out_tokens, float* out_logprobs) {
  using namespace rl;
  if (!logits || !seq_ids || !positions || !sp || !out_tokens || !out_logprobs)
    return (rl_status)set_error(RL_ERR_INVALID_ARG, "rl_sample_logits_static: NULL argument");
  if (vocab < 4 || vocab % 4 || vocab >= (1 << 22))
    return (rl_status)set_error(RL_ERR_INVALID_ARG, "rl_sample_logits_static: vocab %d must be a multiple of 4 in [4, 2^22)", vocab);
  const int n_tiles = (vocab + kSampleTile - 1) / kSampleTile;
  if (n < 1 || n > kStaticRows || (int64_t)n * n_tiles > kStaticTileRows)
    return (rl_status)set_error(RL_ERR_INVALID_ARG,
                                "rl_sample_logits_static: %d rows x %d vocabulary tiles exceed the static scratch "
                                "(at most %d rows and %d row-tiles of %d entries per call)",
                                n, n_tiles, kStaticRows, kStaticTileRows, kSampleTile);
  const int top_k = sp->top_k > (uint32_t)vocab ? 0 : (int)sp->top_k;
  if (sp->temperature > 0.f && sample_is_truncated(vocab, top_k, sp->top_p))
    return (rl_status)set_error(RL_ERR_UNSUPPORTED,
                                "rl_sample_logits_static: top-k / top-p cuts need per-row histograms that the static "
                                "scratch does not hold; use rl_sample_logits");
  unsigned char* base = nullptr;
  hipError_t e = scratch_address(&base);
  if (e != hipSuccess) return (rl_status)set_error(RL_ERR_DEVICE, "rl_sample_logits_static: scratch address: %s", hipGetErrorString(e));
  hipStream_t st = (hipStream_t)stream;
  RowMeta* rows = (RowMeta*)(base + kStaticRowsOff);
  float* forced_z = (float*)(base + kStaticForcedOff);
  float* part = (float*)(base + kStaticPartOff);
  // Nothing has to start at zero: the kernels write every entry they read (all n x n_tiles partials; the forced
  // token's logit whenever the forced id is inside the vocabulary, which is when the second stage reads it).
  static_rows_kernel<<<(n + 255) / 256, 256, 0, st>>>(seq_ids, positions, rows, n);
  launch_sample(st, logits, n, vocab, rows, 0, forced, sp->temperature, sp->seed, part, forced_z, out_tokens, out_logprobs);
  e = hipGetLastError();
  if (e != hipSuccess) return (rl_status)set_error(RL_ERR_DEVICE, "rl_sample_logits_static: %s", hipGetErrorString(e));
  return RL_OK;
}
