// bf16 matrix-core GEMM entry points and the register-staged NT kernel.
//
//  gemm_nt_bf16 / gemm_nn_bf16   C = A * B^T  /  C = A * B  with fused epilogue.  Problems with
//            K % 32 == 0 go to the pipelined direct-to-LDS kernel (gemm_nt_dma.hip); other K % 8 == 0
//            problems to the register-staged kernel below (global -> VGPR -> LDS, padded tiles);
//            anything else to the plain-ALU kernels.
//  gemm_wgrad_bf16               dW[N,K] = G[M,N]^T * A[M,K]: picks the number of token ranges and
//            launches the kernel of gemm_wgrad_dma.hip; the partial tiles of the ranges are summed
//            afterwards in range order, so results do not depend on scheduling.
//
// Register layout of v_mfma_f32_32x32x16_bf16, per lane l of the wavefront:
//   A operand: row l%32, k = 8*(l/32) .. +7;  B operand: column l%32, same k;
//   D: column l%32, rows 8*(v/4) + 4*(l/32) + v%4 for accumulator register v.
#include "mfma.h"

namespace rev {

// ----------------------------------------------------------------------------------------
// epilogues (compile-time kind); m, n are global indices, acc the float32 sum
// ----------------------------------------------------------------------------------------
template <int KIND>
__device__ __forceinline__ void epi_store(const Epi& e, int m, int n, float acc, float biasv) {
    const int64_t idx = (int64_t)m * e.ldo + n;
    if (KIND == EPI_BIAS) {
        reinterpret_cast<bf16*>(e.out)[idx] = __float2bfloat16(acc + biasv);
    } else if (KIND == EPI_BIAS_GELU) {
        float h = acc + biasv;
        if (e.out != nullptr) reinterpret_cast<bf16*>(e.out)[idx] = __float2bfloat16(h);
        reinterpret_cast<bf16*>(e.out2)[idx] = __float2bfloat16(gelu_f(h));
    } else if (KIND == EPI_RESIDUAL) {
        e.outf[idx] = e.res[idx] + e.sign * (acc + biasv);
    } else if (KIND == EPI_GELU_BWD) {
        float h = __bfloat162float(reinterpret_cast<const bf16*>(e.aux)[idx]);
        reinterpret_cast<bf16*>(e.out)[idx] = __float2bfloat16(acc * gelu_grad_f(h));
    } else if (KIND == EPI_PLAIN) {
        reinterpret_cast<bf16*>(e.out)[idx] = __float2bfloat16(acc);
    } else {
        e.outf[idx] = acc;
    }
}

// ----------------------------------------------------------------------------------------
// NT GEMM
// ----------------------------------------------------------------------------------------
constexpr int NT_BK = 64;
constexpr int NT_LDP = NT_BK + 8;     // LDS row pitch in elements (144 B: 16-byte rows land on distinct banks)

template <int BM, int BN, int WM, int WN, int KIND>
__global__ __launch_bounds__(WM * WN * 64) void gemm_nt_kernel(const bf16* __restrict__ A, int64_t lda,
                                                                const bf16* __restrict__ B, int64_t ldb,
                                                                int M, int N, int K, Epi epi) {
    constexpr int NTH = WM * WN * 64;
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    constexpr int CA = BM * (NT_BK / 8) / NTH, CB = BN * (NT_BK / 8) / NTH;
    static_assert(CA * NTH == BM * (NT_BK / 8) && CB * NTH == BN * (NT_BK / 8), "tile/thread mismatch");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    uint16_t* As = reinterpret_cast<uint16_t*>(smem);                 // [2][BM][LDP]
    uint16_t* Bs = As + 2 * BM * NT_LDP;                              // [2][BN][LDP]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int tiles_n = (N + BN - 1) / BN;
    const int tile = xcd_remap(blockIdx.x, gridDim.x);
    const int m0 = (tile / tiles_n) * BM, n0 = (tile % tiles_n) * BN;

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    u32x4_t ra[CA], rb[CB];
    const u32x4_t zero4 = {0u, 0u, 0u, 0u};
#define NT_GLOAD(kt)                                                                                   \
    {                                                                                                  \
        _Pragma("unroll") for (int i = 0; i < CA; ++i) {                                               \
            const int idx = tid + i * NTH, row = idx >> 3, ch = idx & 7;                               \
            const int gk = (kt) * NT_BK + ch * 8;                                                      \
            const int gr = min(m0 + row, M - 1);                                                       \
            ra[i] = (gk < K) ? *reinterpret_cast<const u32x4_t*>(A + (int64_t)gr * lda + gk) : zero4;    \
        }                                                                                              \
        _Pragma("unroll") for (int i = 0; i < CB; ++i) {                                               \
            const int idx = tid + i * NTH, row = idx >> 3, ch = idx & 7;                               \
            const int gk = (kt) * NT_BK + ch * 8;                                                      \
            const int gr = min(n0 + row, N - 1);                                                       \
            rb[i] = (gk < K) ? *reinterpret_cast<const u32x4_t*>(B + (int64_t)gr * ldb + gk) : zero4;    \
        }                                                                                              \
    }
#define NT_LSTORE(buf)                                                                                 \
    {                                                                                                  \
        _Pragma("unroll") for (int i = 0; i < CA; ++i) {                                               \
            const int idx = tid + i * NTH, row = idx >> 3, ch = idx & 7;                               \
            *reinterpret_cast<u32x4_t*>(As + ((buf) * BM + row) * NT_LDP + ch * 8) = ra[i];              \
        }                                                                                              \
        _Pragma("unroll") for (int i = 0; i < CB; ++i) {                                               \
            const int idx = tid + i * NTH, row = idx >> 3, ch = idx & 7;                               \
            *reinterpret_cast<u32x4_t*>(Bs + ((buf) * BN + row) * NT_LDP + ch * 8) = rb[i];              \
        }                                                                                              \
    }

    const int nk = (K + NT_BK - 1) / NT_BK;
    NT_GLOAD(0);
    NT_LSTORE(0);
    __syncthreads();
    const int fr = lane & 31, fk = (lane >> 5) * 8;
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) NT_GLOAD(kt + 1);
        const uint16_t* Ab = As + (buf * BM + wm * TM * 32 + fr) * NT_LDP + fk;
        const uint16_t* Bb = Bs + (buf * BN + wn * TN * 32 + fr) * NT_LDP + fk;
#pragma unroll
        for (int kk = 0; kk < NT_BK / 16; ++kk) {
            bf16x8_t a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) a[i] = *reinterpret_cast<const bf16x8_t*>(Ab + i * 32 * NT_LDP + kk * 16);
#pragma unroll
            for (int j = 0; j < TN; ++j) b[j] = *reinterpret_cast<const bf16x8_t*>(Bb + j * 32 * NT_LDP + kk * 16);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) NT_LSTORE(buf ^ 1);
        __syncthreads();
    }

    // epilogue straight from the accumulator layout
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = n0 + wn * TN * 32 + j * 32 + (lane & 31);
        if (n >= N) continue;
        float biasv = 0.f;
        if (KIND == EPI_BIAS || KIND == EPI_BIAS_GELU || KIND == EPI_RESIDUAL)
            biasv = __bfloat162float(reinterpret_cast<const bf16*>(epi.bias)[n]);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int mb = m0 + wm * TM * 32 + i * 32 + 4 * (lane >> 5);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = mb + 8 * (v >> 2) + (v & 3);
                if (m < M) epi_store<KIND>(epi, m, n, acc[i][j][v], biasv);
            }
        }
    }
}

template <int BM, int BN, int WM, int WN, int KIND>
static int launch_nt(hipStream_t s, const bf16* A, int64_t lda, const bf16* B, int64_t ldb, int M, int N, int K,
                     const Epi& epi) {
    constexpr size_t shmem = (size_t)2 * (BM + BN) * NT_LDP * sizeof(uint16_t);
    static LdsLimit lim;
    auto kern = gemm_nt_kernel<BM, BN, WM, WN, KIND>;
    if (int rc = lim.ensure(reinterpret_cast<const void*>(kern), (int)shmem)) return rc;
    const int tiles = ((M + BM - 1) / BM) * ((N + BN - 1) / BN);
    hipLaunchKernelGGL(kern, dim3(tiles), dim3(WM * WN * 64), shmem, s, A, lda, B, ldb, M, N, K, epi);
    REV_HIP(hipGetLastError());
    return REV_OK;
}

int gemm_bf16_dma(hipStream_t s, const bf16* A, int64_t lda, const bf16* B, int64_t ldb,
                  int M, int N, int K, const Epi& epi, bool b_kmajor);

bool gemm_bf16_fast_path(const bf16* A, int64_t lda, const bf16* B, int64_t ldb, int N, int K, const Epi& epi) {
    const uintptr_t ptrs = (uintptr_t)A | (uintptr_t)B | (uintptr_t)epi.out | (uintptr_t)epi.out2 | (uintptr_t)epi.outf |
                           (uintptr_t)epi.bias | (uintptr_t)epi.res | (uintptr_t)epi.aux;
    return K % 32 == 0 && N % 8 == 0 && (lda & 7) == 0 && (ldb & 7) == 0 && epi.ldo % 4 == 0 && (ptrs & 15) == 0;
}

// C[M,N] = A[M,K] * B[K,N]   (B row-major [K, ldb]): the input-gradient form, weights as stored
int gemm_nn_bf16(hipStream_t s, const bf16* A, int64_t lda, const bf16* B, int64_t ldb,
                 int M, int N, int K, const Epi& epi) {
    if (!gemm_bf16_fast_path(A, lda, B, ldb, N, K, epi)) return gemm_nn_bf16_simple(s, A, lda, B, ldb, M, N, K, epi);
    ProfScope ps(K_GEMM_NT, s, 2.0 * M * N * K);
    return gemm_bf16_dma(s, A, lda, B, ldb, M, N, K, epi, true);
}

int gemm_nt_bf16(hipStream_t s, const bf16* A, int64_t lda, const bf16* B, int64_t ldb,
                 int M, int N, int K, const Epi& epi) {
    if ((lda & 7) || (ldb & 7) || (K & 7) || ((uintptr_t)A & 15) || ((uintptr_t)B & 15)) {
        return gemm_nt_bf16_simple(s, A, lda, B, ldb, M, N, K, epi);
    }
    ProfScope ps(K_GEMM_NT, s, 2.0 * M * N * K);
    if (gemm_bf16_fast_path(A, lda, B, ldb, N, K, epi)) return gemm_bf16_dma(s, A, lda, B, ldb, M, N, K, epi, false);
    switch (epi.kind) {
#define CASE(KIND) case KIND: return launch_nt<128, 128, 2, 2, KIND>(s, A, lda, B, ldb, M, N, K, epi);
        CASE(EPI_BIAS) CASE(EPI_BIAS_GELU) CASE(EPI_RESIDUAL) CASE(EPI_GELU_BWD) CASE(EPI_PLAIN) CASE(EPI_PLAIN_F32)
#undef CASE
    }
    set_error("gemm_nt_bf16: unknown epilogue");
    return REV_EINVAL;
}

// ----------------------------------------------------------------------------------------
// weight gradient: dW[N,K] = sum over tokens m of G[m,n] * A[m,k]
// ----------------------------------------------------------------------------------------
constexpr int WG_BP = 128;            // tile rows (n)
constexpr int WG_BQ = 128;            // tile cols (k)
constexpr int WG_BR = 64;             // tokens per step

// The token reduction is cut into S ranges so that tiles * S fills, but does not exceed, the
// workgroup slots of the chip (256 CUs x 2 resident workgroups): one full round, no ragged second one.
// Narrow layers with very many tokens (window-attention stages: a handful of tiles, thousands of
// steps) get up to 128 ranges; the partial sums stay below 64 MB.
static int wgrad_splits(int M, int N, int K) {
    const int tiles = ((N + WG_BP - 1) / WG_BP) * ((K + WG_BQ - 1) / WG_BQ);
    int S = 512 / tiles;
    const int steps = (M + WG_BR - 1) / WG_BR;
    if (S > steps / 4) S = steps / 4;                          // at least 4 steps per range
    const int64_t cap = ((int64_t)64 << 20) / ((int64_t)N * K * 4);   // at most 64 MB of partial sums
    if (S > cap) S = (int)cap;
    if (S > 128) S = 128;
    if (S < 1) S = 1;
    const int sps = (steps + S - 1) / S;
    return (steps + sps - 1) / sps;                            // no empty ranges
}
int64_t wgrad_partial_elems(int M, int N, int K) {
    const int S = wgrad_splits(M, N, K);
    return S > 1 ? (int64_t)S * N * K : 0;
}

int launch_wgrad_dma(hipStream_t s, const bf16* G, int64_t ldg, const bf16* A, int64_t lda, int M, int N, int K,
                     int S, int sps, float* out);
int launch_wgrad_dma_group(hipStream_t s, WgradGroup grp, int M, int S, int sps);

int gemm_wgrad_bf16(hipStream_t s, const bf16* G, int64_t ldg, const bf16* A, int64_t lda,
                    int M, int N, int K, float* dW, float* partial, int64_t partial_elems, RedSeg* defer) {
    if (defer) defer->P = 0;            // P == 0: nothing left to reduce
    if ((ldg & 7) || (lda & 7) || (N & 7) || (K & 7) || ((uintptr_t)G & 15) || ((uintptr_t)A & 15)) {
        return gemm_wgrad_bf16_simple(s, G, ldg, A, lda, M, N, K, dW);
    }
    const int S = wgrad_splits(M, N, K);
    if (S > 1 && (partial == nullptr || partial_elems < (int64_t)S * N * K)) {
        set_error("gemm_wgrad_bf16: split scratch too small");
        return REV_EWORKSPACE;
    }
    const int steps = (M + WG_BR - 1) / WG_BR;
    const int sps = (steps + S - 1) / S;
    const int tiles = ((N + WG_BP - 1) / WG_BP) * ((K + WG_BQ - 1) / WG_BQ);
    {
        ProfScope ps(K_GEMM_WGRAD, s, 2.0 * M * N * K);
        int rc = launch_wgrad_dma(s, G, ldg, A, lda, M, N, K, S, sps, S > 1 ? partial : dW);
        if (rc) return rc;
    }
    if (S > 1) {
        const RedSeg g = {partial, dW, nullptr, (int64_t)N * K, (int64_t)N * K, (int64_t)N * K, S};
        if (defer) { *defer = g; return REV_OK; }
        return reduce_multi(s, &g, 1);
    }
    return REV_OK;
}

// Token ranges of a group launch: tiles of all items x S fills, but does not exceed, the 512 workgroup slots; at
// least 4 steps per range; at most 64 MB of pieces per item.
int wgrad_group_ranges(int M, const int* N, const int* K, int count) {
    int tiles_total = 0;
    for (int k = 0; k < count; ++k) tiles_total += ((N[k] + WG_BP - 1) / WG_BP) * ((K[k] + WG_BQ - 1) / WG_BQ);
    const int steps = (M + WG_BR - 1) / WG_BR;
    int S = 512 / (tiles_total > 0 ? tiles_total : 1);
    if (S > steps / 4) S = steps / 4;
    if (S > 128) S = 128;
    for (int k = 0; k < count; ++k) {
        const int64_t cap = ((int64_t)64 << 20) / ((int64_t)N[k] * K[k] * 4);
        if (S > cap) S = (int)cap;
    }
    if (S < 1) S = 1;
    const int sps = (steps + S - 1) / S;
    return (steps + sps - 1) / sps;                            // no empty ranges
}

int gemm_wgrad_bf16_group(hipStream_t s, const WgradItem* items, int count, int M, RedSeg* segs, int max_ranges) {
    bool fast = count >= 1 && count <= WGRAD_GROUP_MAX;
    for (int k = 0; k < count && fast; ++k) {
        const WgradItem& it = items[k];
        if ((it.ldg & 7) || (it.lda & 7) || (it.N & 7) || (it.K & 7) || ((uintptr_t)it.G & 15) || ((uintptr_t)it.A & 15))
            fast = false;
    }
    if (!fast) {                          // one at a time (any shape)
        for (int k = 0; k < count; ++k) {
            const WgradItem& it = items[k];
            int rc = gemm_wgrad_bf16(s, it.G, it.ldg, it.A, it.lda, M, it.N, it.K, it.dW, it.partial, it.partial_elems, &segs[k]);
            if (rc) return rc;
        }
        return REV_OK;
    }
    // token ranges: tiles of all items x S fills, but does not exceed, the 512 workgroup slots; at least 4 steps per
    // range; no more ranges than every item's scratch holds
    WgradGroup grp = {};
    grp.count = count;
    int tiles_total = 0;
    double flops = 0;
    for (int k = 0; k < count; ++k) {
        grp.p[k].tile0 = tiles_total;
        tiles_total += ((items[k].N + WG_BP - 1) / WG_BP) * ((items[k].K + WG_BQ - 1) / WG_BQ);
        flops += 2.0 * M * items[k].N * items[k].K;
    }
    grp.tiles_total = tiles_total;
    const int steps = (M + WG_BR - 1) / WG_BR;
    int Ns[WGRAD_GROUP_MAX], Ks[WGRAD_GROUP_MAX];
    for (int k = 0; k < count; ++k) { Ns[k] = items[k].N; Ks[k] = items[k].K; }
    int S = wgrad_group_ranges(M, Ns, Ks, count);
    if (max_ranges > 0 && S > max_ranges) S = max_ranges;
    for (int k = 0; k < count; ++k) {
        const int64_t cap = items[k].partial ? items[k].partial_elems / ((int64_t)items[k].N * items[k].K) : 0;
        if (S > cap) S = (int)cap;
    }
    if (S < 1) S = 1;
    const int sps = (steps + S - 1) / S;
    S = (steps + sps - 1) / sps;                               // no empty ranges
    for (int k = 0; k < count; ++k) {
        const WgradItem& it = items[k];
        const int64_t nk = (int64_t)it.N * it.K;
        grp.p[k].G = it.G; grp.p[k].A = it.A; grp.p[k].ldg = it.ldg; grp.p[k].lda = it.lda;
        grp.p[k].N = it.N; grp.p[k].K = it.K;
        grp.p[k].out = S > 1 ? it.partial : it.dW;
        grp.p[k].split_stride = nk;
        segs[k] = {it.partial, it.dW, nullptr, nk, nk, nk, S > 1 ? S : 0};
    }
    ProfScope ps(K_GEMM_WGRAD, s, flops);
    return launch_wgrad_dma_group(s, grp, M, S, sps);
}

}  // namespace rev
