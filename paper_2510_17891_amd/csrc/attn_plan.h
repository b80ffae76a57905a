// Host-side planning of the decode attention: how a context is cut into segments (shared with the kernels) and
// which rows of a batch can have their leading segments computed once for several rows.
//
// The G samples of one prompt (Section 2.3) hold the prompt's full pages in common.  Rows of such sequences that
// also have the same context length are cut into the same segments, and the segments that lie inside the common
// pages see the same keys and values: they are computed once per set of rows.
#pragma once
#include <stdint.h>

#include <algorithm>
#include <vector>

#if defined(__HIPCC__)
#define RL_HOST_DEVICE __host__ __device__
#else
#define RL_HOST_DEVICE
#endif

namespace rl {

// Segments of a context of ctx keys: their number, and the first 32-key step of segment sgm (n_it = steps of the
// context, n_seg = its segments; sgm <= n_seg <= 256 and n_it < 2^16, so the product fits 32 bits).
RL_HOST_DEVICE inline int attn_num_segments(int ctx) { return 4 * ((ctx + 1023) / 1024); }
RL_HOST_DEVICE inline int attn_seg_begin(int sgm, int n_it, int n_seg) {
  return (int)(((unsigned)sgm * (unsigned)n_it) / (unsigned)n_seg);
}

// Rows of equal context length whose leading pages are the same physical pages: their first n_segs segments are
// computed once for the set.
constexpr int kAttnSetRows = 8;
struct AttnShared {
  int32_t rows[kAttnSetRows];  // entries beyond n_rows repeat rows[0]
  int32_t n_rows;
  int32_t n_segs;
};

// Rows a set may hold: the matrix operand has 16 columns of (row, query head of the kv head) pairs, and the kernel
// for bf16 pages can run two such operands side by side (the one for fp8 pages has the registers for one).  Two
// operands halve the reads of the common keys once more but make the set's blocks the longest of the launch, which
// pays only when the launch is large and bound by memory traffic: from 1024 (row, kv head) pairs on, four row blocks
// per compute unit (measured: a loss at 64 rows, even at 96 to 128 rows, a gain from 128 rows with long prompts on).
// The choice changes no bit of any result.
inline int attn_rows_per_set(int group, bool kv_fp8, int n_rows, int n_kv) {
  const int one_operand = std::min(4, 16 / group);
  if (kv_fp8 || n_rows * n_kv < 1024) return one_operand;
  return std::min(kAttnSetRows, 32 / group);
}

// Leading segments of a context of ctx keys that end inside the first shared_keys keys.
inline int attn_shared_segments(int ctx, int shared_keys) {
  const int n_it = (ctx + 31) >> 5, n_seg = attn_num_segments(ctx);
  int s = 0;
  while (s < n_seg && attn_seg_begin(s + 1, n_it, n_seg) * 32 <= shared_keys) ++s;
  return s;
}

struct AttnPlan {
  std::vector<int32_t> skip;     // per row: leading segments some set covers
  std::vector<AttnShared> sets;
  int max_shared_segs = 0;
};

// prefix_id[i] != 0 names the page-sharing family of row i (equal ids: the first prefix_blocks[i] pages are the
// same physical pages), pos[i] is the row's position.  rows_per_set <= kAttnSetRows.
inline void plan_shared_attention(int n, const int64_t* prefix_id, const int32_t* prefix_blocks, const int32_t* pos,
                                  int rows_per_set, AttnPlan* plan) {
  plan->skip.assign(n, 0);
  plan->sets.clear();
  plan->max_shared_segs = 0;
  std::vector<int> order;
  for (int i = 0; i < n; ++i)
    if (prefix_id[i] != 0) order.push_back(i);
  std::sort(order.begin(), order.end(), [&](int a, int b) {
    if (prefix_id[a] != prefix_id[b]) return prefix_id[a] < prefix_id[b];
    if (pos[a] != pos[b]) return pos[a] < pos[b];
    return a < b;
  });
  size_t i = 0;
  while (i < order.size()) {
    size_t e = i + 1;
    while (e < order.size() && prefix_id[order[e]] == prefix_id[order[i]] && pos[order[e]] == pos[order[i]]) ++e;
    const int first = order[i];
    const int shared_keys = std::min(prefix_blocks[first] * 16, pos[first]);  // a row's own key is never shared
    const int segs = attn_shared_segments(pos[first] + 1, shared_keys);
    if (segs > 0) {
      for (size_t b = i; b + 1 < e; b += rows_per_set) {  // a single left-over row computes everything itself
        AttnShared s;
        s.n_rows = (int)std::min<size_t>(rows_per_set, e - b);
        s.n_segs = segs;
        for (int k = 0; k < kAttnSetRows; ++k) s.rows[k] = order[b + (k < s.n_rows ? k : 0)];
        for (int k = 0; k < s.n_rows; ++k) plan->skip[order[b + k]] = segs;
        plan->sets.push_back(s);
        plan->max_shared_segs = std::max(plan->max_shared_segs, segs);
      }
    }
    i = e;
  }
}

// Rows that feed consecutive positions of one sequence (prefill, scoring).  Positions inside one aligned window of
// 32 have the same number of 32-key steps and hence the same segments, and every row's keys are a prefix of the
// keys of the row after it: up to rows_per_set (<= kAttnSetRows) neighbouring rows of a window form a set that computes ALL their
// segments side by side (n_segs = every segment, each column masked at its own context length), so the window's
// keys are read once per set instead of once per row.  rows[0] of a set is its highest position (the block takes
// its page list and step count from it).  seq[i], pos[i]: sequence and position of row i; rows of a sequence must
// be adjacent and ascending, as the chunks of a prefill are.
inline void plan_window_sets(int n, const int32_t* seq, const int32_t* pos, int rows_per_set, AttnPlan* plan) {
  plan->skip.assign(n, 0);
  plan->sets.clear();
  plan->max_shared_segs = 0;
  int i = 0;
  while (i < n) {
    int e = i + 1;
    while (e < n && e - i < rows_per_set && seq[e] == seq[i] && pos[e] == pos[e - 1] + 1 && (pos[e] >> 5) == (pos[i] >> 5)) ++e;
    if (e - i >= 2) {
      AttnShared s;
      s.n_rows = e - i;
      s.n_segs = attn_num_segments(pos[e - 1] + 1);  // the same for every member
      for (int k = 0; k < kAttnSetRows; ++k) s.rows[k] = e - 1 - (k < s.n_rows ? k : 0);
      for (int k = i; k < e; ++k) plan->skip[k] = s.n_segs;
      plan->sets.push_back(s);
      plan->max_shared_segs = std::max(plan->max_shared_segs, s.n_segs);
    }
    i = e;
  }
}

}  // namespace rl
