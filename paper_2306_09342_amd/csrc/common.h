// Internal declarations shared by the translation units of librevstack.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_bf16.h>
#include <stdint.h>
#include <string>
#include <cmath>
#include <atomic>

#include "rev_stack.h"

namespace rev {

typedef __hip_bfloat16 bf16;

// ---- error plumbing -------------------------------------------------------
void set_error(const std::string& msg);
int  hip_fail(hipError_t e, const char* what, const char* file, int line);

#define REV_HIP(expr)                                                        \
    do {                                                                     \
        hipError_t _e = (expr);                                              \
        if (_e != hipSuccess) return ::rev::hip_fail(_e, #expr, __FILE__, __LINE__); \
    } while (0)

// Raises a kernel's dynamic-LDS limit once per process.  Callable from several host threads: the runtime call is
// idempotent and the flag is published only after it has succeeded, so whoever finds it set may launch.
struct LdsLimit {
    std::atomic<bool> done{false};
    int ensure(const void* kern, int bytes) {
        if (done.load(std::memory_order_acquire)) return 0;
        hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
        if (e != hipSuccess) return hip_fail(e, "hipFuncSetAttribute(MaxDynamicSharedMemorySize)", __FILE__, __LINE__);
        done.store(true, std::memory_order_release);
        return 0;
    }
};

// ---- kernel families for the per-family timing ------------------------------
enum Kind {
    K_GEMM_NT = 0,   // activation x weight^T contractions (forward/recompute and dgrad)
    K_GEMM_WGRAD,    // weight-gradient contractions (long reduction over tokens)
    K_ATTN_FWD,
    K_ATTN_BWD,
    K_LN_FWD,
    K_LN_BWD,
    K_COLSUM,        // bias gradients (column sums), first stage
    K_REDUCE,        // fixed-order second stage of column sums / split reductions
    K_CONVERT,       // dtype conversion
    K_OPTIM,         // optimizer update
    K_COUNT
};

// Brackets a launch with events when profiling is on; otherwise nothing.
struct ProfScope {
    ProfScope(Kind k, hipStream_t s, double work);
    ~ProfScope();
    Kind kind; hipStream_t stream; void* rec;
};
bool profiling();

// AdamW update of n packed elements (optimizer.hip)
int adamw_step(hipStream_t s, int64_t n, float* master, void* params_bf16, const float* grad, float* m, float* v,
               int step, float lr, float beta1, float beta2, float eps, float weight_decay);
// plain SGD update of n packed elements (optimizer.hip)
int sgd_step(hipStream_t s, int64_t n, float* master, void* params_bf16, const float* grad, float lr);

// ---- small device helpers ------------------------------------------------------
__device__ __forceinline__ float to_f(float v) { return v; }
__device__ __forceinline__ float to_f(bf16 v) { return __bfloat162float(v); }
template <typename T> __device__ __forceinline__ T from_f(float v);
template <> __device__ __forceinline__ float from_f<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_f<bf16>(float v) { return __float2bfloat16(v); }

// Sum over the 64 lanes, result in every lane.  Rotations inside each row of 16 lanes are DPP
// modifiers of the add itself (no LDS round trip); the four row sums are then read out as scalars.
// The order of the additions is fixed.
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}
__device__ __forceinline__ float wave_sum(float v) {
    v += dpp_mov<0x128>(v);    // row_ror:8
    v += dpp_mov<0x124>(v);    // row_ror:4
    v += dpp_mov<0x122>(v);    // row_ror:2
    v += dpp_mov<0x121>(v);    // row_ror:1
    const float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
    const float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
    const float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
    return (r0 + r1) + (r2 + r3);
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// exact GELU and its derivative (erf form)
__device__ __forceinline__ float gelu_f(float x) {
    return 0.5f * x * (1.0f + erff(x * 0.70710678118654752f));
}
__device__ __forceinline__ float gelu_grad_f(float x) {
    float cdf = 0.5f * (1.0f + erff(x * 0.70710678118654752f));
    float pdf = 0.39894228040143268f * __expf(-0.5f * x * x);
    return cdf + x * pdf;
}

// One fixed-order column reduction, described so that several of them can share a launch:
// out[i] = sum over p = 0..P-1 (ascending) of partial[p * stride + i] for i < n; elements [0, split) go to
// `out`, elements [split, n) to `out2` (dropped if out2 is null).
struct RedSeg {
    const float* partial;
    float* out;
    float* out2;
    int64_t stride, n, split;
    int P;
};
constexpr int RED_MAX_SEGS = 6;
// All segments in one launch (every length a multiple of 4, nseg <= RED_MAX_SEGS).
int reduce_multi(hipStream_t s, const RedSeg* segs, int nseg);

// ---- epilogue description shared by the GEMM launchers ----------------------------
enum EpiKind {
    EPI_BIAS = 0,      // out = acc + bias[n]                               (out: act type)
    EPI_BIAS_GELU,     // h = acc + bias[n]; out = h (skipped when out is null); out2 = gelu(h)   (act type)
    EPI_RESIDUAL,      // outf = res[m,n] + sign * (acc + bias[n])          (float32)
    EPI_GELU_BWD,      // out = acc * gelu'(aux[m,n])                       (act type)
    EPI_PLAIN,         // out = acc                                         (act type)
    EPI_PLAIN_F32      // outf = acc                                        (float32)
};

struct Epi {
    int kind;
    void* out;          // act-typed output  [M, ldo]
    void* out2;         // second act-typed output (gelu)
    float* outf;        // float32 output
    const void* bias;   // parameter-typed [N]
    const float* res;   // float32 [M, ldo]
    const void* aux;    // act-typed [M, ldo] (pre-activation for GELU backward)
    float sign;
    int64_t ldo;
    float* colsum;      // EPI_GELU_BWD, matrix-core path: per-row-strip column sums of the output,
                        // [gemm_colsum_rows(M)][N] float32 (nullable)
    bool solo;          // the launch runs alone on the device (one stream): the tile shape may be chosen
                        // to fill the chip by itself; results do not depend on it
};
// 64-row strips of column-sum partials the matrix-core GEMM writes for M rows, and an upper bound for sizing
int gemm_colsum_strips(int M);
inline int gemm_colsum_strips_max(int M) { return ((M + 255) / 256) * 4; }

// C[M,N] (+epilogue) = A[M,K] * B[N,K]^T.  A, B row-major with leading dims lda, ldb.
// fp32 flavour: A, B float.  bf16 flavour: A, B bf16.
int gemm_nt_f32(hipStream_t s, const float* A, int64_t lda, const float* B, int64_t ldb,
                int M, int N, int K, const Epi& epi);
int gemm_nt_bf16(hipStream_t s, const bf16* A, int64_t lda, const bf16* B, int64_t ldb,
                 int M, int N, int K, const Epi& epi);
// C[M,N] = A[M,K] * B[K,N]  (B row-major [K, ldb]): the input-gradient form, weights as stored.
int gemm_nn_bf16(hipStream_t s, const bf16* A, int64_t lda, const bf16* B, int64_t ldb,
                 int M, int N, int K, const Epi& epi);
// true when the pipelined matrix-core kernel (the one that honours Epi::colsum) takes this problem
bool gemm_bf16_fast_path(const bf16* A, int64_t lda, const bf16* B, int64_t ldb, int N, int K, const Epi& epi);
int gemm_nn_bf16_simple(hipStream_t s, const bf16* A, int64_t lda, const bf16* B, int64_t ldb,
                        int M, int N, int K, const Epi& epi);
int gemm_nn_f32(hipStream_t s, const float* A, int64_t lda, const float* B, int64_t ldb,
                int M, int N, int K, const Epi& epi);
// dW[N,K] (float32, ld = K) = G[M,N]^T * A[M,K]  -- reduction over the M tokens.
// `partial` is scratch for the fixed-order split of the reduction (may be unused).
int gemm_wgrad_f32(hipStream_t s, const float* G, int64_t ldg, const float* A, int64_t lda,
                   int M, int N, int K, float* dW, float* partial, int64_t partial_elems, RedSeg* defer = nullptr);
int gemm_wgrad_bf16(hipStream_t s, const bf16* G, int64_t ldg, const bf16* A, int64_t lda,
                    int M, int N, int K, float* dW, float* partial, int64_t partial_elems, RedSeg* defer = nullptr);

// Several weight gradients over the same M tokens in ONE launch (the four of a transformer block): together their
// tiles fill the device, so the token range is cut into fewer pieces (none for Rev-ViT-B) than each would need alone.
// segs[k] receives the deferred fixed-order reduction of item k's pieces (P == 0: nothing to reduce).
constexpr int WGRAD_GROUP_MAX = 4;
struct WgradItem {
    const bf16* G; int64_t ldg;        // cotangent [M, N]
    const bf16* A; int64_t lda;        // activation [M, K]
    int N, K;
    float* dW;                         // [N, K]
    float* partial; int64_t partial_elems;   // scratch for the pieces (may be null / 0: then this item allows no cut)
};
// max_ranges > 0 caps the number of token ranges (1: never cut, whatever share of the device the tiles fill).
int gemm_wgrad_bf16_group(hipStream_t s, const WgradItem* items, int count, int M, RedSeg* segs, int max_ranges = 0);
// token ranges the group launch uses for these shapes (1: no pieces, no scratch); item k then needs ranges * N[k] * K[k]
// floats of scratch
int wgrad_group_ranges(int M, const int* N, const int* K, int count);
// device-side description of the launch (gemm_wgrad_dma.hip)
struct WgradProblem { const bf16* G; const bf16* A; float* out; int64_t ldg, lda, split_stride; int N, K, tile0; };
struct WgradGroup { WgradProblem p[WGRAD_GROUP_MAX]; int count, tiles_total; };

// plain vector-ALU flavours (also the fall-back for shapes the matrix-core kernels do not take)
int gemm_nt_bf16_simple(hipStream_t s, const bf16* A, int64_t lda, const bf16* B, int64_t ldb,
                        int M, int N, int K, const Epi& epi);
int gemm_wgrad_bf16_simple(hipStream_t s, const bf16* G, int64_t ldg, const bf16* A, int64_t lda,
                           int M, int N, int K, float* dW);
template <typename T>
int attention_forward_simple(hipStream_t s, const T* qkv, T* o, float* lse, int B, int T_, int H, int dh,
                             const int* key_len = nullptr);
template <typename T>
int attention_backward_simple(hipStream_t s, const T* qkv, const T* o, const T* dout, const float* lse,
                              T* dqkv, float* delta, int B, int T_, int H, int dh, const int* key_len = nullptr);

// ---- memory-bound kernels ---------------------------------------------------------
// y = LN(x; g, b), stats[2*row] = mean, stats[2*row+1] = rstd
template <typename TA, typename TP>
int ln_forward(hipStream_t s, const float* x, const TP* g, const TP* b, float eps,
               TA* y, float* stats, int M, int D);
// out = r + LNbwd(dn; x, stats, g);  outb (nullable) = act-typed copy of out;
// dgb[0:D] = d gamma, dgb[D:2D] = d beta, dbias[D] (nullable) = column sums of out;
// all three float32, summed in a fixed order via `partial` (>= ln_bwd_partial_elems floats)
template <typename TA, typename TP>
int ln_backward(hipStream_t s, const TA* dn, const float* x, const float* stats, const TP* g,
                const float* r, float* out, TA* outb, float* dgb, float* dbias,
                float* partial, int M, int D, RedSeg* defer = nullptr);
int64_t ln_bwd_partial_elems(int M, int D);

// out[n] = sum_m in[m, n]   (float32 out, fixed summation order).  With `defer` the second stage is not
// launched: its description is returned for a later reduce_multi.
template <typename T>
int colsum(hipStream_t s, const T* in, int64_t ld, int M, int N, float* out, float* partial, RedSeg* defer = nullptr);
int64_t colsum_partial_elems(int M, int N);

int convert_f32_to_bf16(hipStream_t s, const float* in, bf16* out, int64_t n);

// ---- attention ----------------------------------------------------------------------
// qkv [B*T, 3D] (q|k|v, head-major inside each), o [B*T, D], lse [B, H, T].
// key_len (nullable, device, [B]): key-padding mask -- the keys at positions >= key_len[b] (clamped to
// [1, T]) of sample b are left out of every softmax of that sample; all T query rows are computed.
template <typename TA>
int attention_forward(hipStream_t s, const TA* qkv, TA* o, float* lse, int B, int T, int H, int dh,
                      const int* key_len = nullptr);
template <typename TA>
int attention_backward(hipStream_t s, const TA* qkv, const TA* o, const TA* dout, const float* lse,
                       TA* dqkv, float* delta, int B, int T, int H, int dh, const int* key_len = nullptr,
                       bool solo = false);     // solo: the launch has the device to itself (one stream)

}  // namespace rev
