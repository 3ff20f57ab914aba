// Optimizer update of a training step: AdamW (Adam with decoupled weight decay), the optimizer the
// paper's throughput experiments train with (Sec. 4).  One pass over the packed parameter vector:
// float32 master weights, float32 moments and the float32 gradient in, master weights and moments
// out, plus (bf16 mode) the bf16 copy the stack's kernels read.  Purely HBM-bound: 16 bytes read and
// 12 (14) written per element, nothing reused, so the kernel is a grid-stride loop of 16-byte accesses.
#include "common.h"

namespace rev {

typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));

struct AdamwArgs {
    float beta1, beta2, one_minus_beta1, one_minus_beta2;
    float inv_bc1, inv_bc2;        // 1 / (1 - beta^t), computed in double on the host
    float lr, eps, weight_decay;
};

__device__ __forceinline__ float adamw_one(float& th, float g, float& m, float& v, const AdamwArgs& a) {
    m = a.beta1 * m + a.one_minus_beta1 * g;
    v = a.beta2 * v + a.one_minus_beta2 * g * g;
    const float mhat = m * a.inv_bc1;
    const float vhat = v * a.inv_bc2;
    th = th - a.lr * (mhat / (sqrtf(vhat) + a.eps) + a.weight_decay * th);
    return th;
}

template <bool BF16OUT>
__global__ __launch_bounds__(256) void adamw_kernel(int64_t n, float* __restrict__ master, __bf16* __restrict__ pout,
                                                    const float* __restrict__ grad, float* __restrict__ m,
                                                    float* __restrict__ v, AdamwArgs a) {
    const int64_t n4 = n >> 2;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) {
        f32x4_t th = reinterpret_cast<const f32x4_t*>(master)[i];
        const f32x4_t g = reinterpret_cast<const f32x4_t*>(grad)[i];
        f32x4_t mm = reinterpret_cast<const f32x4_t*>(m)[i];
        f32x4_t vv = reinterpret_cast<const f32x4_t*>(v)[i];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            float t = th[k], m1 = mm[k], v1 = vv[k];
            adamw_one(t, g[k], m1, v1, a);
            th[k] = t; mm[k] = m1; vv[k] = v1;
        }
        reinterpret_cast<f32x4_t*>(master)[i] = th;
        reinterpret_cast<f32x4_t*>(m)[i] = mm;
        reinterpret_cast<f32x4_t*>(v)[i] = vv;
        if (BF16OUT) {
            bf16x4_t b;
#pragma unroll
            for (int k = 0; k < 4; ++k) b[k] = (__bf16)th[k];          // round to nearest even
            reinterpret_cast<bf16x4_t*>(pout)[i] = b;
        }
    }
    // the up-to-3 elements behind the last full group of 4
    const int64_t tail = (n4 << 2) + (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (blockIdx.x == 0 && tail < n) {
        float t = master[tail], m1 = m[tail], v1 = v[tail];
        adamw_one(t, grad[tail], m1, v1, a);
        master[tail] = t; m[tail] = m1; v[tail] = v1;
        if (BF16OUT) pout[tail] = (__bf16)t;
    }
}

// Plain stochastic gradient descent, theta -= lr * g (the paper reports the same behaviour with it):
// 8 bytes read and 4 (6) written per element.
template <bool BF16OUT>
__global__ __launch_bounds__(256) void sgd_kernel(int64_t n, float* __restrict__ master, __bf16* __restrict__ pout,
                                                  const float* __restrict__ grad, float lr) {
    const int64_t n4 = n >> 2;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) {
        f32x4_t th = reinterpret_cast<const f32x4_t*>(master)[i];
        const f32x4_t g = reinterpret_cast<const f32x4_t*>(grad)[i];
#pragma unroll
        for (int k = 0; k < 4; ++k) th[k] = th[k] - lr * g[k];
        reinterpret_cast<f32x4_t*>(master)[i] = th;
        if (BF16OUT) {
            bf16x4_t b;
#pragma unroll
            for (int k = 0; k < 4; ++k) b[k] = (__bf16)th[k];
            reinterpret_cast<bf16x4_t*>(pout)[i] = b;
        }
    }
    const int64_t tail = (n4 << 2) + (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (blockIdx.x == 0 && tail < n) {
        const float t = master[tail] - lr * grad[tail];
        master[tail] = t;
        if (BF16OUT) pout[tail] = (__bf16)t;
    }
}

int sgd_step(hipStream_t s, int64_t n, float* master, void* params_bf16, const float* grad, float lr) {
    const int64_t n4 = n >> 2;
    int64_t blocks = (n4 + 255) / 256;
    if (blocks > 256 * 16) blocks = 256 * 16;
    if (blocks < 1) blocks = 1;
    ProfScope ps(K_OPTIM, s, (double)n * (params_bf16 ? 14.0 : 12.0));
    if (params_bf16)
        hipLaunchKernelGGL(sgd_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, s, n, master,
                           reinterpret_cast<__bf16*>(params_bf16), grad, lr);
    else
        hipLaunchKernelGGL(sgd_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, s, n, master, (__bf16*)nullptr, grad, lr);
    REV_HIP(hipGetLastError());
    return REV_OK;
}

int adamw_step(hipStream_t s, int64_t n, float* master, void* params_bf16, const float* grad, float* m, float* v,
               int step, float lr, float beta1, float beta2, float eps, float weight_decay) {
    AdamwArgs a;
    a.beta1 = beta1; a.beta2 = beta2;
    a.one_minus_beta1 = (float)(1.0 - (double)beta1);
    a.one_minus_beta2 = (float)(1.0 - (double)beta2);
    a.inv_bc1 = (float)(1.0 / (1.0 - std::pow((double)beta1, (double)step)));
    a.inv_bc2 = (float)(1.0 / (1.0 - std::pow((double)beta2, (double)step)));
    a.lr = lr; a.eps = eps; a.weight_decay = weight_decay;
    const int64_t n4 = n >> 2;
    int64_t blocks = (n4 + 255) / 256;
    if (blocks > 256 * 16) blocks = 256 * 16;       // 16 workgroups per CU, grid-stride beyond
    if (blocks < 1) blocks = 1;
    ProfScope ps(K_OPTIM, s, (double)n * (params_bf16 ? 30.0 : 28.0));
    if (params_bf16) {
        hipLaunchKernelGGL(adamw_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, s, n, master,
                           reinterpret_cast<__bf16*>(params_bf16), grad, m, v, a);
    } else {
        hipLaunchKernelGGL(adamw_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, s, n, master,
                           (__bf16*)nullptr, grad, m, v, a);
    }
    REV_HIP(hipGetLastError());
    return REV_OK;
}

}  // namespace rev
