// Forward value of the policy objective with Hierarchical Reward Decomposition (Section 2.3) and of its
// uniform-reward GRPO counterpart (Appendix C), over a batch of n_prompts groups of G sampled outputs.
//
// One block per output: group-mean baselines from the G rewards of its group, plan/code split (given, or found
// as the first delimiter token), then a fixed-order sum over its tokens of the clipped-ratio terms.  A second
// one-block kernel adds the per-output terms in index order, so the value is reproducible bit for bit.
#include <hip/hip_runtime.h>

#include "../../include/rl.h"
#include "device_utils.h"
#include "kernels.h"

namespace rl {

namespace {

__device__ __forceinline__ float block_sum_256(float v, float* sh) {
  v = wave_sum(v);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  const float r = (sh[0] + sh[1]) + (sh[2] + sh[3]);
  __syncthreads();
  return r;
}

__global__ __launch_bounds__(256) void objective_seq_kernel(int G, const int32_t* __restrict__ off,
                                                            const int32_t* __restrict__ n_plan_in,
                                                            const int32_t* __restrict__ tokens, int delimiter,
                                                            const float* __restrict__ lp_new,
                                                            const float* __restrict__ lp_old,
                                                            const float* __restrict__ r_speedup,
                                                            const float* __restrict__ r_correct, float alpha, float eps,
                                                            float beta, int mode, float* __restrict__ seq_term,
                                                            int32_t* __restrict__ n_plan_out) {
  __shared__ float sh[4];
  __shared__ int sh_first;
  const int k = blockIdx.x, i = k / G;
  const int begin = off[k], len = off[k + 1] - begin;
  // group baselines (G is small; every thread does the same sums in the same order)
  float mean_s = 0.f, mean_c = 0.f, mean_u = 0.f;
  for (int j = 0; j < G; ++j) {
    const float rs = r_speedup[i * G + j], rc = r_correct[i * G + j];
    mean_s += rs;
    mean_c += rc;
    mean_u += beta * rc + (1.0f - beta) * rs;
  }
  mean_s /= (float)G; mean_c /= (float)G; mean_u /= (float)G;
  const float a_plan = r_speedup[k] - mean_s, a_code = r_correct[k] - mean_c;
  const float a_uni = beta * r_correct[k] + (1.0f - beta) * r_speedup[k] - mean_u;
  // plan length: given, or up to and including the first delimiter (whole output if there is none)
  int n_plan;
  if (n_plan_in != nullptr) {
    n_plan = min(max(n_plan_in[k], 0), len);  // a count outside the output is read as "none" / "all of it"
  } else {
    if (threadIdx.x == 0) sh_first = len;
    __syncthreads();
    for (int t = threadIdx.x; t < len; t += 256)
      if (tokens[begin + t] == delimiter) atomicMin(&sh_first, t + 1);
    __syncthreads();
    n_plan = sh_first;
  }
  if (n_plan_out != nullptr && threadIdx.x == 0) n_plan_out[k] = n_plan;
  float acc = 0.f;
  for (int t = threadIdx.x; t < len; t += 256) {
    const float s = expf(lp_new[begin + t] - lp_old[begin + t]);
    const float sc = fminf(fmaxf(s, 1.0f - eps), 1.0f + eps);
    if (mode == 0) {
      const bool plan = t < n_plan;
      const float A = plan ? a_plan : a_code;
      const float term = fminf(A * s, A * sc);
      acc += plan ? alpha * term : term;
    } else {
      acc += a_uni * fminf(s, sc);
    }
  }
  acc = block_sum_256(acc, sh);
  if (threadIdx.x == 0) seq_term[k] = len > 0 ? acc / (float)len : 0.f;
}

// J = mean over prompts of the mean over the group = sum of all terms / (n_prompts * G); one block, fixed order.
__global__ __launch_bounds__(256) void objective_reduce_kernel(const float* __restrict__ seq_term, int n, float* __restrict__ out) {
  __shared__ float sh[4];
  float acc = 0.f;
  for (int k = threadIdx.x; k < n; k += 256) acc += seq_term[k];
  acc = block_sum_256(acc, sh);
  if (threadIdx.x == 0) *out = acc / (float)n;
}

}  // namespace

}  // namespace rl

extern "C" rl_status rl_hrd_objective(void* stream, int32_t n_prompts, int32_t group_size, const int32_t* offsets,
                                      const int32_t* n_plan, const int32_t* tokens, int32_t delimiter_token,
                                      const float* lp_new, const float* lp_old, const float* r_speedup,
                                      const float* r_correct, const rl_objective_params* p, float* seq_terms,
                                      int32_t* n_plan_out, float* out_value) {
  if (n_prompts < 1 || group_size < 1 || (int64_t)n_prompts * group_size > (1 << 24))
    return (rl_status)rl::set_error(RL_ERR_INVALID_ARG, "rl_hrd_objective: n_prompts %d x group_size %d outside [1, 2^24]",
                                    n_prompts, group_size);
  if (!offsets || !lp_new || !lp_old || !r_speedup || !r_correct || !p || !seq_terms || !out_value)
    return (rl_status)rl::set_error(RL_ERR_INVALID_ARG, "rl_hrd_objective: NULL argument");
  if (!n_plan && !tokens)
    return (rl_status)rl::set_error(RL_ERR_INVALID_ARG, "rl_hrd_objective: neither n_plan nor tokens given");
  if (p->mode != 0 && p->mode != 1)
    return (rl_status)rl::set_error(RL_ERR_INVALID_ARG, "rl_hrd_objective: mode %d is neither 0 (HRD) nor 1 (uniform)", p->mode);
  hipStream_t st = (hipStream_t)stream;
  const int n = n_prompts * group_size;
  rl::objective_seq_kernel<<<n, 256, 0, st>>>(group_size, offsets, n_plan, tokens, delimiter_token, lp_new, lp_old,
                                              r_speedup, r_correct, p->alpha, p->eps_clip, p->beta, p->mode, seq_terms,
                                              n_plan_out);
  rl::objective_reduce_kernel<<<1, 256, 0, st>>>(seq_terms, n, out_value);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return (rl_status)rl::set_error(RL_ERR_DEVICE, "rl_hrd_objective: %s", hipGetErrorString(e));
  return RL_OK;
}
