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

// Alg. 1, second loop, with every density of the step known (the exact form: the mean density of
// a layer still to come is that layer's own density of this step).  grid (batch); thread j =
// layer j sums the densities behind it (from the last layer down), thread 0 then hands out the
// budget layer by layer: B^l = Theta^l / (Theta^l + R^l) * B_kv, B_kv -= B^l, and E^l = B^l
// rounded half up, at least 1, at most k_cap.
__global__ __launch_bounds__(kMaxLayers) void cutoff_budgets_kernel(int n_layers, int batch, float k_mean, int k_cap,
                                                                    const float* __restrict__ theta,
                                                                    float* __restrict__ budget,
                                                                    int32_t* __restrict__ count,
                                                                    float* __restrict__ budget_left) {
  __shared__ float th[kMaxLayers], rest[kMaxLayers];
  const int s = blockIdx.x, j = threadIdx.x;
  if (j < n_layers) th[j] = theta[size_t(j) * batch + s];
  __syncthreads();
  if (j < n_layers) {
    float r = 0.f;
    for (int i = n_layers - 1; i > j; --i) r += th[i];
    rest[j] = r;
  }
  __syncthreads();
  if (j == 0) {
    float b_kv = float(n_layers) * k_mean;
    for (int l = 0; l < n_layers; ++l) {
      const float den = th[l] + rest[l];
      const float b_l = den > 0.f ? th[l] / den * b_kv : b_kv;
      b_kv -= b_l;
      budget[size_t(l) * batch + s] = b_l;
      count[size_t(l) * batch + s] = int(fminf(fmaxf(floorf(b_l + 0.5f), 1.f), float(k_cap)));
    }
    if (budget_left != nullptr) budget_left[s] = b_kv;
  }
}

int launch_cutoff_budgets(int batch, int n_layers, float k_mean, int k_cap, const float* theta, float* budget,
                          int32_t* count, float* budget_left, hipStream_t stream) {
  const int threads = (n_layers + 63) / 64 * 64;
  hipLaunchKernelGGL(cutoff_budgets_kernel, dim3(batch), dim3(threads), 0, stream, n_layers, batch, k_mean, k_cap,
                     theta, budget, count, budget_left);
  return hip_status("cutoff_budgets");
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
