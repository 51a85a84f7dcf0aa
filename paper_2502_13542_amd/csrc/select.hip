// Information density, per-layer budget and block selection
// (Sec. 4.2, Eq. (11), Eq. (12); Alg. 1, second and third loop): one workgroup of 16
// wavefronts per sequence runs the selection step.
#include "common.h"
#include "launch.h"
#include "select_body.h"

namespace actqkv {

constexpr int kSelectThreads = 1024;

__global__ __launch_bounds__(kSelectThreads) void select_kernel(
    const float* __restrict__ scores, int64_t score_stride, int nb_capacity, int nb_begin,
    const int32_t* __restrict__ nb_end, int k_cap, int flags, float* __restrict__ budget_remaining,
    const float* __restrict__ theta_rest_sum, int32_t* __restrict__ idx, int32_t* __restrict__ n_sel,
    float* __restrict__ theta_out, float* __restrict__ budget_out) {
  __shared__ SelectLds<kSelectThreads> lds;
  const int s = blockIdx.x, tid = threadIdx.x;
  const float* sc_mem = scores + size_t(s) * score_stride + nb_begin;
  // the row has nb_capacity entries whatever nb_end says
  const ScoreRow<kSelectThreads> sc{sc_mem, tid < nb_capacity - nb_begin ? sc_mem[tid] : 0.f};
  // clamped from both sides before anything is computed from it: a huge negative value in
  // device memory must not wrap around in the subtraction
  const int end = min(max(nb_end[s], nb_begin), nb_capacity);
  const int n = max(end - nb_begin, 0);
  SelectIo io{budget_remaining, theta_rest_sum, budget_remaining, idx, n_sel, theta_out, budget_out, true};
  io.density_only = (flags & ACTQKV_SELECT_DENSITY_ONLY) != 0;
  // E^l given: it is read from n_sel (thread 0 reads it before it writes the clamped value back)
  if (flags & ACTQKV_SELECT_GIVEN_COUNT) io.count_in = n_sel;
  select_body<kSelectThreads>(sc, s, n, nb_begin, k_cap, (flags & ACTQKV_SELECT_ENTROPY_TOPK) != 0, io, lds);
}

int launch_select(int batch, const float* scores, int64_t score_stride, int nb_capacity, int nb_begin,
                  const int32_t* nb_end, int k_cap, int flags, float* budget_remaining,
                  const float* theta_rest_sum, int32_t* idx, int32_t* n_sel, float* theta,
                  float* budget, hipStream_t stream) {
  hipLaunchKernelGGL(select_kernel, dim3(batch), dim3(kSelectThreads), 0, stream, scores,
                     score_stride, nb_capacity, nb_begin, nb_end, k_cap, flags, budget_remaining,
                     theta_rest_sum, idx, n_sel, theta, budget);
  return hip_status("select");
}

}  // namespace actqkv
