// C wrappers around the host sequence table so that its logic can be exercised without a GPU.
// Built with g++ into its own small library by the CPU tests; not part of the product library.
#include "attn_plan.h"
#include "seq_table.h"
#include "weight_order.h"

extern "C" {

void* st_create(int max_seqs, int max_ctx, long long n_pages) { return new rl::SeqTable(max_seqs, max_ctx, n_pages); }
void st_destroy(void* t) { delete (rl::SeqTable*)t; }
long long st_free_pages(void* t) { return ((rl::SeqTable*)t)->free_pages(); }
int st_active(void* t, int s) { return ((rl::SeqTable*)t)->active(s) ? 1 : 0; }
int st_len(void* t, int s) { return ((rl::SeqTable*)t)->len(s); }
int st_pages_missing(void* t, int s, int tokens) { return ((rl::SeqTable*)t)->pages_missing(s, tokens); }
void st_activate(void* t, int s) { ((rl::SeqTable*)t)->activate(s); }
void st_set_len(void* t, int s, int n) { ((rl::SeqTable*)t)->set_len(s, n); }
void st_release(void* t, int s) { ((rl::SeqTable*)t)->release(s); }
void st_shuffle(void* t, unsigned long long seed) { ((rl::SeqTable*)t)->shuffle_free(seed); }
void st_share_prefix(void* t, int dst, int src, int n_blocks) { ((rl::SeqTable*)t)->share_prefix(dst, src, n_blocks); }
int st_refcount(void* t, int page) { return ((rl::SeqTable*)t)->refcount(page); }
int st_n_seq_pages(void* t, int s) { return (int)((rl::SeqTable*)t)->pages(s).size(); }
int st_seq_page(void* t, int s, int i) { return ((rl::SeqTable*)t)->pages(s)[i]; }
// returns the number of grants written (seq, block, page triples)
int st_reserve(void* t, int s, int tokens, int* grants_out, int max_grants) {
  std::vector<rl::PageGrant> g;
  ((rl::SeqTable*)t)->reserve(s, tokens, &g);
  int n = 0;
  for (auto& x : g) {
    if (n >= max_grants) break;
    grants_out[3 * n] = x.seq; grants_out[3 * n + 1] = x.block; grants_out[3 * n + 2] = x.page;
    ++n;
  }
  return (int)g.size();
}

long long st_prefix_id(void* t, int s) { return ((rl::SeqTable*)t)->prefix_id(s); }
int st_prefix_blocks(void* t, int s) { return ((rl::SeqTable*)t)->prefix_blocks(s); }
int st_weight_kb_slot(int kb, int seg) { return rl::weight_kb_slot(kb, seg); }
int st_attn_rows_per_set(int group, int kv_fp8, int n_rows, int n_kv) {
  return rl::attn_rows_per_set(group, kv_fp8 != 0, n_rows, n_kv);
}
int st_attn_num_segments(int ctx) { return rl::attn_num_segments(ctx); }
int st_attn_seg_begin(int sgm, int ctx) { return rl::attn_seg_begin(sgm, (ctx + 31) >> 5, rl::attn_num_segments(ctx)); }
// plan of one decode batch: skip_out[n]; sets_out gets (rows[8], n_rows, n_segs) per set; returns the number of sets
int st_plan_shared(void* t, int n, const int* seq_ids, const int* pos, int rows_per_set, int* skip_out, int* sets_out,
                   int max_sets) {
  auto* T = (rl::SeqTable*)t;
  std::vector<int64_t> fam(n);
  std::vector<int32_t> blocks(n);
  for (int i = 0; i < n; ++i) { fam[i] = T->prefix_id(seq_ids[i]); blocks[i] = T->prefix_blocks(seq_ids[i]); }
  rl::AttnPlan plan;
  rl::plan_shared_attention(n, fam.data(), blocks.data(), pos, rows_per_set, &plan);
  for (int i = 0; i < n; ++i) skip_out[i] = plan.skip[i];
  for (size_t k = 0; k < plan.sets.size() && (int)k < max_sets; ++k) {
    for (int e = 0; e < rl::kAttnSetRows; ++e) sets_out[10 * k + e] = plan.sets[k].rows[e];
    sets_out[10 * k + 8] = plan.sets[k].n_rows;
    sets_out[10 * k + 9] = plan.sets[k].n_segs;
  }
  return (int)plan.sets.size();
}

int st_plan_windows(int n, const int* seq, const int* pos, int rows_per_set, int* skip_out, int* sets_out, int max_sets) {
  rl::AttnPlan plan;
  rl::plan_window_sets(n, seq, pos, rows_per_set, &plan);
  for (int i = 0; i < n; ++i) skip_out[i] = plan.skip[i];
  for (size_t k = 0; k < plan.sets.size() && (int)k < max_sets; ++k) {
    for (int e = 0; e < rl::kAttnSetRows; ++e) sets_out[10 * k + e] = plan.sets[k].rows[e];
    sets_out[10 * k + 8] = plan.sets[k].n_rows;
    sets_out[10 * k + 9] = plan.sets[k].n_segs;
  }
  return (int)plan.sets.size();
}

}  // extern "C"
