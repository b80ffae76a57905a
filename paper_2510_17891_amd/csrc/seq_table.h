// Host-side sequence table and KV page allocator (no GPU calls; unit-tested on the CPU).
//
// A page holds 16 tokens of K and V for every layer.  Pages are handed out from a LIFO free list; a call
// that needs several pages first checks that all of them exist, so a failing call changes nothing.
// Pages are reference counted: the samples of one prompt share the pages that the prompt fills completely
// (they are never written again), and a page returns to the free list when its last holder is released.
// Placement: a growing sequence first tries the page right after its last one (inside an aligned run of kRun
// pages), and fresh requests are served run starts first, so that sequences growing in lock step still end up
// with long physically contiguous stretches (fewer TLB entries and DRAM rows per streamed context).
#pragma once
#include <stdint.h>

#include <algorithm>
#include <vector>

namespace rl {

struct PageGrant {
  int32_t seq, block, page;
};

class SeqTable {
 public:
  static constexpr int kBlock = 16;
  static constexpr int kRun = 32;  // pages per placement run (512 tokens)

  SeqTable(int max_seqs, int max_ctx, int64_t n_pages)
      : max_seqs_(max_seqs), max_ctx_(max_ctx), max_blocks_(max_ctx / kBlock), n_pages_(n_pages),
        len_(max_seqs, -1), pages_(max_seqs), prefix_id_(max_seqs, 0), prefix_blocks_(max_seqs, 0),
        ref_(n_pages, 0), is_free_(n_pages, 1), free_count_(n_pages) {
    free_.reserve(2 * n_pages);
    // popped from the back: run starts first (0, kRun, 2 kRun, ...), then the remaining pages in ascending order
    for (int64_t p = n_pages - 1; p >= 0; --p)
      if (p % kRun != 0) free_.push_back((int32_t)p);
    for (int64_t p = (n_pages - 1) / kRun * kRun; p >= 0; p -= kRun) free_.push_back((int32_t)p);
  }

  int max_seqs() const { return max_seqs_; }
  int max_ctx() const { return max_ctx_; }
  int max_blocks() const { return max_blocks_; }
  int64_t n_pages() const { return n_pages_; }
  int64_t free_pages() const { return free_count_; }

  bool valid_id(int32_t s) const { return s >= 0 && s < max_seqs_; }
  bool active(int32_t s) const { return valid_id(s) && len_[s] >= 0; }
  int32_t len(int32_t s) const { return len_[s]; }
  const std::vector<int32_t>& pages(int32_t s) const { return pages_[s]; }

  static int blocks_for(int tokens) { return (tokens + kBlock - 1) / kBlock; }

  // Pages still missing for `s` to hold `tokens` tokens (s may be inactive: then all of them).
  int pages_missing(int32_t s, int tokens) const {
    int have = len_[s] >= 0 ? (int)pages_[s].size() : 0;
    return std::max(0, blocks_for(tokens) - have);
  }

  // Activate a fresh sequence with length 0.
  void activate(int32_t s) {
    len_[s] = 0;
    pages_[s].clear();
    prefix_id_[s] = 0;
    prefix_blocks_[s] = 0;
  }

  // Grow the page list of `s` to cover `tokens` tokens; the caller has checked free_pages().
  void reserve(int32_t s, int tokens, std::vector<PageGrant>* grants) {
    int need = blocks_for(tokens);
    while ((int)pages_[s].size() < need) {
      const int32_t p = take_page(pages_[s].empty() ? -1 : pages_[s].back());
      ref_[p] = 1;
      if (grants) grants->push_back(PageGrant{s, (int32_t)pages_[s].size(), p});
      pages_[s].push_back(p);
    }
  }

  void set_len(int32_t s, int32_t n) { len_[s] = n; }

  void release(int32_t s) {
    for (auto it = pages_[s].rbegin(); it != pages_[s].rend(); ++it)
      if (--ref_[*it] == 0) give_page(*it);
    pages_[s].clear();
    len_[s] = -1;
  }

  // Make the (freshly activated, page-less) sequence `dst` share the first `n_blocks` pages of `src`.
  // Both then carry the same family id: sequences with equal ids hold the same first prefix_blocks() pages.
  void share_prefix(int32_t dst, int32_t src, int n_blocks) {
    for (int b = 0; b < n_blocks; ++b) {
      const int32_t p = pages_[src][b];
      ++ref_[p];
      pages_[dst].push_back(p);
    }
    if (n_blocks > 0) {
      if (prefix_id_[src] == 0 || prefix_blocks_[src] != n_blocks) {
        prefix_id_[src] = ++next_prefix_id_;
        prefix_blocks_[src] = n_blocks;
      }
      prefix_id_[dst] = prefix_id_[src];
      prefix_blocks_[dst] = n_blocks;
    }
  }
  int64_t prefix_id(int32_t s) const { return prefix_id_[s]; }
  int32_t prefix_blocks(int32_t s) const { return prefix_blocks_[s]; }
  int32_t refcount(int32_t page) const { return ref_[page]; }

  // Deterministic shuffle of the free list (test aid: results must not depend on page placement).
  void shuffle_free(uint64_t seed) {
    compact();
    contiguous_ = false;  // scattered placement is the point of this aid
    uint64_t x = seed * 0x9E3779B97F4A7C15ull + 0x7F4A7C15ull;
    for (size_t i = free_.size(); i > 1; --i) {
      x ^= x << 13; x ^= x >> 7; x ^= x << 17;
      std::swap(free_[i - 1], free_[x % i]);
    }
  }

 private:
  // The stack may hold entries of pages that were meanwhile taken by the "next page" rule (or twice after a
  // take/give cycle); is_free_ is the truth and stale entries are skipped when popped.
  int32_t take_page(int32_t last) {
    if (contiguous_ && last >= 0 && (last + 1) % kRun != 0 && last + 1 < n_pages_ && is_free_[last + 1]) {
      is_free_[last + 1] = 0;
      --free_count_;
      return last + 1;
    }
    for (;;) {
      const int32_t p = free_.back();
      free_.pop_back();
      if (is_free_[p]) {
        is_free_[p] = 0;
        --free_count_;
        return p;
      }
    }
  }
  void give_page(int32_t p) {
    is_free_[p] = 1;
    ++free_count_;
    if ((int64_t)free_.size() >= 4 * n_pages_) compact();
    free_.push_back(p);
  }
  void compact() {  // drop stale and duplicate entries, keeping the pop order of the survivors
    std::vector<char> seen(n_pages_, 0);
    std::vector<int32_t> keep;
    keep.reserve(free_.size());
    for (auto it = free_.rbegin(); it != free_.rend(); ++it)
      if (is_free_[*it] && !seen[*it]) { seen[*it] = 1; keep.push_back(*it); }
    free_.assign(keep.rbegin(), keep.rend());
  }

  int max_seqs_, max_ctx_, max_blocks_;
  int64_t n_pages_;
  std::vector<int32_t> len_;  // -1 = inactive
  std::vector<std::vector<int32_t>> pages_;
  std::vector<int64_t> prefix_id_;  // 0 = shares nothing
  std::vector<int32_t> prefix_blocks_;
  int64_t next_prefix_id_ = 0;
  std::vector<int32_t> free_;
  std::vector<int32_t> ref_;  // holders per page
  std::vector<char> is_free_;
  int64_t free_count_;
  bool contiguous_ = true;
};

}  // namespace rl
