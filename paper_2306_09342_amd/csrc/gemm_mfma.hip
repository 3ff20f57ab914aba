// bf16 matrix-core GEMMs (placeholder dispatch: plain kernels until the MFMA path lands)
#include "common.h"
namespace rev {
int64_t wgrad_partial_elems(int M, int N, int K) { (void)M; (void)N; (void)K; return 64; }
int gemm_nt_bf16(hipStream_t s, const bf16* A, int64_t lda, const bf16* B, int64_t ldb,
                 int M, int N, int K, const Epi& epi) {
    return gemm_nt_bf16_simple(s, A, lda, B, ldb, M, N, K, epi);
}
int gemm_wgrad_bf16(hipStream_t s, const bf16* G, int64_t ldg, const bf16* A, int64_t lda,
                    int M, int N, int K, float* dW, float*, int64_t) {
    return gemm_wgrad_bf16_simple(s, G, ldg, A, lda, M, N, K, dW);
}
template <typename TA>
int attention_forward(hipStream_t s, const TA* qkv, TA* o, float* lse, int B, int T, int H, int dh) {
    return attention_forward_simple<TA>(s, qkv, o, lse, B, T, H, dh);
}
template <typename TA>
int attention_backward(hipStream_t s, const TA* qkv, const TA* o, const TA* dout, const float* lse,
                       TA* dqkv, float* delta, int B, int T, int H, int dh) {
    return attention_backward_simple<TA>(s, qkv, o, dout, lse, dqkv, delta, B, T, H, dh);
}
template int attention_forward<float>(hipStream_t, const float*, float*, float*, int, int, int, int);
template int attention_forward<bf16>(hipStream_t, const bf16*, bf16*, float*, int, int, int, int);
template int attention_backward<float>(hipStream_t, const float*, const float*, const float*, const float*, float*, float*, int, int, int, int);
template int attention_backward<bf16>(hipStream_t, const bf16*, const bf16*, const bf16*, const float*, bf16*, float*, int, int, int, int);
}
