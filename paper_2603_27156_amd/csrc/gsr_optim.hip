// Parameter updates that turn gsr_step (forward + inverse + backward) into a full training step
// (Section 5 trains for 250 epochs; the paper does not name its optimiser): plain SGD with weight
// decay, and Adam with bias correction as Kingma & Ba define it.  Element-wise, float32, in place.
#include "gsr_internal.h"

#include <algorithm>
#include <cmath>

namespace gsr {

__global__ __launch_bounds__(256) void k_sgd(int64_t count, float* __restrict__ w, const float* __restrict__ dw, float lr,
                                             float wd) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (int64_t)gridDim.x * blockDim.x) {
        const float x = w[i];
        w[i] = x - lr * (dw[i] + wd * x);
    }
}

// m = b1 m + (1 - b1) g;  v = b2 v + (1 - b2) g^2;  w -= lr * (m / c1) / (sqrt(v / c2) + eps),  g = dw + wd w,
// c1 = 1 - b1^t, c2 = 1 - b2^t (computed on the host in double precision)
__global__ __launch_bounds__(256) void k_adam(int64_t count, float* __restrict__ w, const float* __restrict__ dw,
                                              float* __restrict__ m, float* __restrict__ v, float lr, float b1, float b2,
                                              float eps, float wd, float inv_c1, float inv_c2) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (int64_t)gridDim.x * blockDim.x) {
        const float x = w[i];
        const float g = dw[i] + wd * x;
        const float mi = b1 * m[i] + (1.0f - b1) * g;
        const float vi = b2 * v[i] + (1.0f - b2) * g * g;
        m[i] = mi;
        v[i] = vi;
        w[i] = x - lr * (mi * inv_c1) / (sqrtf(vi * inv_c2) + eps);
    }
}

static unsigned update_blocks(int64_t count) { return (unsigned)std::min<int64_t>((count + 255) / 256, 16384); }

}  // namespace gsr

using namespace gsr;

extern "C" {

gsr_status_t gsr_sgd_update(float* w, const float* dw, int64_t count, float lr, float weight_decay, void* stream) {
    if (count < 0) return fail(GSR_ERR_INVALID_ARG, "negative count");
    if (count == 0) return GSR_OK;
    if (!w || !dw) return fail(GSR_ERR_INVALID_ARG, "null pointer");
    hipLaunchKernelGGL(k_sgd, dim3(update_blocks(count)), dim3(256), 0, (hipStream_t)stream, count, w, dw, lr, weight_decay);
    GSR_HIP_CHECK(hipGetLastError());
    return GSR_OK;
}

gsr_status_t gsr_adam_update(float* w, const float* dw, float* m, float* v, int64_t count, int64_t t, float lr, float beta1,
                             float beta2, float eps, float weight_decay, void* stream) {
    if (count < 0) return fail(GSR_ERR_INVALID_ARG, "negative count");
    if (t < 1) return fail(GSR_ERR_INVALID_ARG, "Adam's step counter starts at 1");
    if (!(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f)) return fail(GSR_ERR_INVALID_ARG, "beta outside [0,1)");
    if (count == 0) return GSR_OK;
    if (!w || !dw || !m || !v) return fail(GSR_ERR_INVALID_ARG, "null pointer");
    const double c1 = 1.0 - std::pow((double)beta1, (double)t), c2 = 1.0 - std::pow((double)beta2, (double)t);
    hipLaunchKernelGGL(k_adam, dim3(update_blocks(count)), dim3(256), 0, (hipStream_t)stream, count, w, dw, m, v, lr, beta1, beta2,
                       eps, weight_decay, (float)(1.0 / c1), (float)(1.0 / c2));
    GSR_HIP_CHECK(hipGetLastError());
    return GSR_OK;
}

}  // extern "C"
