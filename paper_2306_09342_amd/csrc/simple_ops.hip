// Plain vector-ALU kernels: an LDS-tiled GEMM in float32 arithmetic and a
// wavefront-per-row softmax attention (forward and backward).  They carry the
// float32 mode, whose configs are launch-latency bound, and any shape the
// matrix-core kernels do not take.  Every sum has a fixed order.
#include "common.h"

namespace rev {

// ---- epilogue, one element at a time ----------------------------------------------
template <typename T>
__device__ __forceinline__ void apply_epi(const Epi& e, int m, int n, float acc) {
    const int64_t idx = (int64_t)m * e.ldo + n;
    switch (e.kind) {
        case EPI_BIAS:
            reinterpret_cast<T*>(e.out)[idx] = from_f<T>(acc + to_f(reinterpret_cast<const T*>(e.bias)[n]));
            break;
        case EPI_BIAS_GELU: {
            float h = acc + to_f(reinterpret_cast<const T*>(e.bias)[n]);
            if (e.out != nullptr) reinterpret_cast<T*>(e.out)[idx] = from_f<T>(h);
            reinterpret_cast<T*>(e.out2)[idx] = from_f<T>(gelu_f(h));
            break;
        }
        case EPI_RESIDUAL:
            e.outf[idx] = e.res[idx] + e.sign * (acc + to_f(reinterpret_cast<const T*>(e.bias)[n]));
            break;
        case EPI_GELU_BWD:
            reinterpret_cast<T*>(e.out)[idx] = from_f<T>(acc * gelu_grad_f(to_f(reinterpret_cast<const T*>(e.aux)[idx])));
            break;
        case EPI_PLAIN:
            reinterpret_cast<T*>(e.out)[idx] = from_f<T>(acc);
            break;
        default:  // EPI_PLAIN_F32
            e.outf[idx] = acc;
            break;
    }
}

// C[i,j] = sum_k A'(i,k) * B'(k,j)
//   A'(i,k) = TA ? A[k*lda + i] : A[i*lda + k]
//   B'(k,j) = TB ? B[j*ldb + k] : B[k*ldb + j]
// 64x64 tile, 16-deep steps, 256 threads, 4x4 outputs per thread.
template <typename T, bool TA, bool TB>
__global__ __launch_bounds__(256) void gemm_simple_kernel(const T* __restrict__ A, int64_t lda,
                                                          const T* __restrict__ B, int64_t ldb,
                                                          int M, int N, int K, Epi epi) {
    __shared__ float As[16][64 + 4];
    __shared__ float Bs[16][64 + 4];
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += 16) {
        for (int e = tid; e < 64 * 16; e += 256) {
            int i, k;
            if (TA) { i = e & 63; k = e >> 6; } else { k = e & 15; i = e >> 4; }
            int gi = m0 + i, gk = k0 + k;
            float v = 0.f;
            if (gi < M && gk < K) v = to_f(TA ? A[(int64_t)gk * lda + gi] : A[(int64_t)gi * lda + gk]);
            As[k][i] = v;
        }
        for (int e = tid; e < 64 * 16; e += 256) {
            int j, k;
            if (TB) { k = e & 15; j = e >> 4; } else { j = e & 63; k = e >> 6; }
            int gj = n0 + j, gk = k0 + k;
            float v = 0.f;
            if (gj < N && gk < K) v = to_f(TB ? B[(int64_t)gj * ldb + gk] : B[(int64_t)gk * ldb + gj]);
            Bs[k][j] = v;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Bs[k][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
            if (m < M && n < N) apply_epi<T>(epi, m, n, acc[i][j]);
        }
}

template <typename T, bool TA, bool TB>
static int launch_simple(hipStream_t s, Kind kind, const T* A, int64_t lda, const T* B, int64_t ldb,
                         int M, int N, int K, const Epi& epi) {
    ProfScope ps(kind, s, 2.0 * M * N * K);
    dim3 grid((N + 63) / 64, (M + 63) / 64), block(256);
    hipLaunchKernelGGL((gemm_simple_kernel<T, TA, TB>), grid, block, 0, s, A, lda, B, ldb, M, N, K, epi);
    REV_HIP(hipGetLastError());
    return REV_OK;
}

int gemm_nt_f32(hipStream_t s, const float* A, int64_t lda, const float* B, int64_t ldb,
                int M, int N, int K, const Epi& epi) {
    return launch_simple<float, false, true>(s, K_GEMM_NT, A, lda, B, ldb, M, N, K, epi);
}
int gemm_nn_f32(hipStream_t s, const float* A, int64_t lda, const float* B, int64_t ldb,
                int M, int N, int K, const Epi& epi) {
    return launch_simple<float, false, false>(s, K_GEMM_NT, A, lda, B, ldb, M, N, K, epi);
}
int gemm_nt_bf16_simple(hipStream_t s, const bf16* A, int64_t lda, const bf16* B, int64_t ldb,
                        int M, int N, int K, const Epi& epi) {
    return launch_simple<bf16, false, true>(s, K_GEMM_NT, A, lda, B, ldb, M, N, K, epi);
}
int gemm_nn_bf16_simple(hipStream_t s, const bf16* A, int64_t lda, const bf16* B, int64_t ldb,
                        int M, int N, int K, const Epi& epi) {
    return launch_simple<bf16, false, false>(s, K_GEMM_NT, A, lda, B, ldb, M, N, K, epi);
}
int gemm_wgrad_f32(hipStream_t s, const float* G, int64_t ldg, const float* A, int64_t lda,
                   int M, int N, int K, float* dW, float*, int64_t, RedSeg* defer) {
    if (defer) defer->P = 0;
    Epi e = {};
    e.kind = EPI_PLAIN_F32; e.outf = dW; e.ldo = K;
    // dW[n,k] = sum_m G[m,n] * A[m,k]
    return launch_simple<float, true, false>(s, K_GEMM_WGRAD, G, ldg, A, lda, N, K, M, e);
}
int gemm_wgrad_bf16_simple(hipStream_t s, const bf16* G, int64_t ldg, const bf16* A, int64_t lda,
                           int M, int N, int K, float* dW) {
    Epi e = {};
    e.kind = EPI_PLAIN_F32; e.outf = dW; e.ldo = K;
    return launch_simple<bf16, true, false>(s, K_GEMM_WGRAD, G, ldg, A, lda, N, K, M, e);
}

// ---- attention, one wavefront per query (or key) row ------------------------------------------
// Head h of token row t: q at qkv[t, h*dh], k at qkv[t, D + h*dh], v at qkv[t, 2D + h*dh].
template <typename T>
__global__ __launch_bounds__(256) void attn_fwd_simple(const T* __restrict__ qkv, T* __restrict__ o,
                                                       float* __restrict__ lse, const int* __restrict__ key_len,
                                                       int T_, int H, int dh) {
    __shared__ float qs[4][128];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int bh = blockIdx.y, b = bh / H, h = bh % H;
    const int i = blockIdx.x * 4 + wave;
    const int D = H * dh;
    const int64_t ld = 3 * (int64_t)D;
    const float scale = rsqrtf((float)dh);
    const T* base = qkv + (int64_t)b * T_ * ld + h * dh;
    const bool live = i < T_;
    if (live)
        for (int d = lane; d < dh; d += 64) qs[wave][d] = to_f(base[(int64_t)i * ld + d]);
    __syncthreads();
    if (!live) return;
    // key-padding mask: keys at positions >= Tk take no part in the softmax
    const int Tk = key_len ? min(max(key_len[b], 1), T_) : T_;
    float m = -INFINITY, l = 0.f, acc[2] = {0.f, 0.f};
    for (int j0 = 0; j0 < Tk; j0 += 64) {
        const int j = j0 + lane;
        float s = -INFINITY;
        if (j < Tk) {
            const T* kr = base + (int64_t)j * ld + D;
            float dot = 0.f;
            for (int d = 0; d < dh; ++d) dot += qs[wave][d] * to_f(kr[d]);
            s = dot * scale;
        }
        const float mn = fmaxf(m, wave_max(s));
        const float p = (j < Tk) ? __expf(s - mn) : 0.f;
        const float corr = __expf(m - mn);
        l = l * corr + wave_sum(p);
        acc[0] *= corr; acc[1] *= corr;
        m = mn;
        const int cnt = min(64, Tk - j0);
        for (int jj = 0; jj < cnt; ++jj) {
            const float pj = __shfl(p, jj, 64);
            const T* vr = base + (int64_t)(j0 + jj) * ld + 2 * D;
            if (lane < dh) acc[0] += pj * to_f(vr[lane]);
            if (lane + 64 < dh) acc[1] += pj * to_f(vr[lane + 64]);
        }
    }
    T* orow = o + ((int64_t)b * T_ + i) * D + h * dh;
    if (lane < dh) orow[lane] = from_f<T>(acc[0] / l);
    if (lane + 64 < dh) orow[lane + 64] = from_f<T>(acc[1] / l);
    if (lane == 0) lse[(int64_t)bh * T_ + i] = m + __logf(l);
}

// dQ rows and delta_i = sum_d dO[i,d] * O[i,d]
template <typename T>
__global__ __launch_bounds__(256) void attn_bwd_dq_simple(const T* __restrict__ qkv, const T* __restrict__ o,
                                                          const T* __restrict__ dout, const float* __restrict__ lse,
                                                          T* __restrict__ dqkv, float* __restrict__ delta,
                                                          const int* __restrict__ key_len, int T_, int H, int dh) {
    __shared__ float qs[4][128];
    __shared__ float dos[4][128];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int bh = blockIdx.y, b = bh / H, h = bh % H;
    const int i = blockIdx.x * 4 + wave;
    const int D = H * dh;
    const int64_t ld = 3 * (int64_t)D;
    const float scale = rsqrtf((float)dh);
    const T* base = qkv + (int64_t)b * T_ * ld + h * dh;
    const bool live = i < T_;
    float dl = 0.f;
    if (live) {
        const int64_t orow = ((int64_t)b * T_ + i) * D + h * dh;
        for (int d = lane; d < dh; d += 64) {
            float dv = to_f(dout[orow + d]);
            qs[wave][d] = to_f(base[(int64_t)i * ld + d]);
            dos[wave][d] = dv;
            dl += dv * to_f(o[orow + d]);
        }
    }
    __syncthreads();
    if (!live) return;
    dl = wave_sum(dl);
    const float L = lse[(int64_t)bh * T_ + i];
    if (lane == 0) delta[(int64_t)bh * T_ + i] = dl;
    const int Tk = key_len ? min(max(key_len[b], 1), T_) : T_;
    float acc[2] = {0.f, 0.f};
    for (int j0 = 0; j0 < Tk; j0 += 64) {
        const int j = j0 + lane;
        float ds = 0.f;
        if (j < Tk) {
            const T* kr = base + (int64_t)j * ld + D;
            const T* vr = base + (int64_t)j * ld + 2 * D;
            float dot = 0.f, dp = 0.f;
            for (int d = 0; d < dh; ++d) {
                dot += qs[wave][d] * to_f(kr[d]);
                dp += dos[wave][d] * to_f(vr[d]);
            }
            const float p = __expf(dot * scale - L);
            ds = p * (dp - dl) * scale;
        }
        const int cnt = min(64, Tk - j0);
        for (int jj = 0; jj < cnt; ++jj) {
            const float dj = __shfl(ds, jj, 64);
            const T* kr = base + (int64_t)(j0 + jj) * ld + D;
            if (lane < dh) acc[0] += dj * to_f(kr[lane]);
            if (lane + 64 < dh) acc[1] += dj * to_f(kr[lane + 64]);
        }
    }
    T* dq = dqkv + ((int64_t)b * T_ + i) * ld + h * dh;
    if (lane < dh) dq[lane] = from_f<T>(acc[0]);
    if (lane + 64 < dh) dq[lane + 64] = from_f<T>(acc[1]);
}

// dK and dV rows (one wavefront per key row j)
template <typename T>
__global__ __launch_bounds__(256) void attn_bwd_dkv_simple(const T* __restrict__ qkv, const T* __restrict__ dout,
                                                           const float* __restrict__ lse, const float* __restrict__ delta,
                                                           T* __restrict__ dqkv, const int* __restrict__ key_len,
                                                           int T_, int H, int dh) {
    __shared__ float ks[4][128];
    __shared__ float vs[4][128];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int bh = blockIdx.y, b = bh / H, h = bh % H;
    const int j = blockIdx.x * 4 + wave;
    const int D = H * dh;
    const int64_t ld = 3 * (int64_t)D;
    const float scale = rsqrtf((float)dh);
    const T* base = qkv + (int64_t)b * T_ * ld + h * dh;
    const T* dob = dout + (int64_t)b * T_ * D + h * dh;
    const bool live = j < T_;
    if (live)
        for (int d = lane; d < dh; d += 64) {
            ks[wave][d] = to_f(base[(int64_t)j * ld + D + d]);
            vs[wave][d] = to_f(base[(int64_t)j * ld + 2 * D + d]);
        }
    __syncthreads();
    if (!live) return;
    float dk[2] = {0.f, 0.f}, dv[2] = {0.f, 0.f};
    for (int i0 = 0; i0 < T_; i0 += 64) {
        const int i = i0 + lane;
        float p = 0.f, ds = 0.f;
        if (i < T_) {
            const T* qr = base + (int64_t)i * ld;
            const T* dr = dob + (int64_t)i * D;
            float dot = 0.f, dp = 0.f;
            for (int d = 0; d < dh; ++d) {
                dot += to_f(qr[d]) * ks[wave][d];
                dp += to_f(dr[d]) * vs[wave][d];
            }
            p = __expf(dot * scale - lse[(int64_t)bh * T_ + i]);
            ds = p * (dp - delta[(int64_t)bh * T_ + i]) * scale;
        }
        const int cnt = min(64, T_ - i0);
        for (int ii = 0; ii < cnt; ++ii) {
            const float pi = __shfl(p, ii, 64), di = __shfl(ds, ii, 64);
            const T* qr = base + (int64_t)(i0 + ii) * ld;
            const T* dr = dob + (int64_t)(i0 + ii) * D;
            if (lane < dh) { dv[0] += pi * to_f(dr[lane]); dk[0] += di * to_f(qr[lane]); }
            if (lane + 64 < dh) { dv[1] += pi * to_f(dr[lane + 64]); dk[1] += di * to_f(qr[lane + 64]); }
        }
    }
    if (key_len && j >= min(max(key_len[b], 1), T_)) {          // a masked key: no query looked at it
        dk[0] = dk[1] = dv[0] = dv[1] = 0.f;
    }
    T* dkr = dqkv + ((int64_t)b * T_ + j) * ld + D + h * dh;
    T* dvr = dkr + D;
    if (lane < dh) { dkr[lane] = from_f<T>(dk[0]); dvr[lane] = from_f<T>(dv[0]); }
    if (lane + 64 < dh) { dkr[lane + 64] = from_f<T>(dk[1]); dvr[lane + 64] = from_f<T>(dv[1]); }
}

template <typename T>
int attention_forward_simple(hipStream_t s, const T* qkv, T* o, float* lse, int B, int T_, int H, int dh, const int* key_len) {
    ProfScope ps(K_ATTN_FWD, s, 4.0 * B * H * (double)T_ * T_ * dh);
    dim3 grid((T_ + 3) / 4, B * H), block(256);
    hipLaunchKernelGGL((attn_fwd_simple<T>), grid, block, 0, s, qkv, o, lse, key_len, T_, H, dh);
    REV_HIP(hipGetLastError());
    return REV_OK;
}
template <typename T>
int attention_backward_simple(hipStream_t s, const T* qkv, const T* o, const T* dout, const float* lse,
                              T* dqkv, float* delta, int B, int T_, int H, int dh, const int* key_len) {
    ProfScope ps(K_ATTN_BWD, s, 8.0 * B * H * (double)T_ * T_ * dh);
    dim3 grid((T_ + 3) / 4, B * H), block(256);
    hipLaunchKernelGGL((attn_bwd_dq_simple<T>), grid, block, 0, s, qkv, o, dout, lse, dqkv, delta, key_len, T_, H, dh);
    hipLaunchKernelGGL((attn_bwd_dkv_simple<T>), grid, block, 0, s, qkv, dout, lse, delta, dqkv, key_len, T_, H, dh);
    REV_HIP(hipGetLastError());
    return REV_OK;
}
template int attention_forward_simple<float>(hipStream_t, const float*, float*, float*, int, int, int, int, const int*);
template int attention_forward_simple<bf16>(hipStream_t, const bf16*, bf16*, float*, int, int, int, int, const int*);
template int attention_backward_simple<float>(hipStream_t, const float*, const float*, const float*, const float*, float*, float*, int, int, int, int, const int*);
template int attention_backward_simple<bf16>(hipStream_t, const bf16*, const bf16*, const bf16*, const float*, bf16*, float*, int, int, int, int, const int*);

}  // namespace rev
