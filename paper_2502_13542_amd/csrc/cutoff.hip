// Dynamic cut-off across layers and steps (Sec. 4.2, Eq. (12); Alg. 1, second loop):
//   B^l = Theta^l / (Theta^l + sum_{j>l} mean Theta^j) * B_kv,  B_kv <- B_kv - B^l,
// B_kv starting at L * k in every step.  The layers after l have not been computed when layer
// l takes its share (layer l+1's query depends on layer l's output), so their densities enter
// as the running means over the steps so far.  This kernel keeps that history on the device:
// once per step it folds the densities of the step before into (sum, count), and writes the
// step's initial budget and, for every layer, the sum of the mean densities of the layers
// after it - the two cut-off inputs of actqkv_select.
#include "common.h"
#include "launch.h"

namespace actqkv {

constexpr int kMaxLayers = 1024;

// grid (batch); one workgroup per sequence, thread j = layer j.
__global__ __launch_bounds__(kMaxLayers) void cutoff_next_step_kernel(
    int n_layers, int batch, float k_mean, float theta_prior, const float* __restrict__ theta_prev,
    float* __restrict__ theta_sum, float* __restrict__ n_steps, float* __restrict__ budget_remaining,
    float* __restrict__ theta_rest_sum) {
  __shared__ float mean[kMaxLayers];
  const int s = blockIdx.x, j = threadIdx.x;
  const float count = n_steps[s] + (theta_prev != nullptr ? 1.f : 0.f);
  if (j < n_layers) {
    float sum = theta_sum[size_t(s) * n_layers + j];
    if (theta_prev != nullptr) {
      sum += theta_prev[size_t(j) * batch + s];
      theta_sum[size_t(s) * n_layers + j] = sum;
    }
    mean[j] = count > 0.f ? sum / count : theta_prior;
  }
  __syncthreads();
  if (j < n_layers) {
    float rest = 0.f;
    for (int i = n_layers - 1; i > j; --i) rest += mean[i];     // from the last layer down: fixed order
    theta_rest_sum[size_t(j) * batch + s] = rest;
  }
  if (j == 0) {
    n_steps[s] = count;
    budget_remaining[s] = float(n_layers) * k_mean;
  }
}

int launch_cutoff_next_step(int batch, int n_layers, float k_mean, float theta_prior,
                            const float* theta_prev, float* theta_sum, float* n_steps,
                            float* budget_remaining, float* theta_rest_sum, hipStream_t stream) {
  const int threads = (n_layers + 63) / 64 * 64;
  hipLaunchKernelGGL(cutoff_next_step_kernel, dim3(batch), dim3(threads), 0, stream, n_layers, batch,
                     k_mean, theta_prior, theta_prev, theta_sum, n_steps, budget_remaining, theta_rest_sum);
  return hip_status("cutoff_next_step");
}

}  // namespace actqkv
