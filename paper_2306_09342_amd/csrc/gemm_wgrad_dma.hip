// Weight gradient, pipelined flavour:  dW[N,K] = sum over tokens m of G[m,n] * A[m,k].
//
// Both operands have the reduction index (the token) as their slow index.  Their
// tiles -- 64 tokens x 128 columns -- go HBM -> LDS with direct-to-LDS loads in
// the layout they have in memory, and the matrix-core fragments (8 consecutive
// tokens of one column per lane) are gathered with the LDS transpose read, so
// nothing is transposed in memory or in registers.
//
// LDS tile: rows of 128 bf16 (256 B), dense; the 16-byte chunk c of token row r
// sits at position c ^ (4 * (r & 3)).  One transpose read touches 4 consecutive
// token rows x 64 bytes per 32 lanes; the swizzle spreads those 4 rows over
// the 4 quarters of the bank space.
//
// Tokens beyond M and columns beyond N / K are fetched from a block of zeros.
#include "mfma.h"
#include <type_traits>

namespace rev {

constexpr int WD_BP = 128, WD_BQ = 128, WD_BR = 64;
constexpr int WD_TILE = WD_BR * 256;            // bytes of one operand tile
constexpr int WD_STAGE = 2 * WD_TILE;

// One 128 x 128 tile of dW over one token range: `tile` counts the tiles of this weight gradient, `split` its token
// ranges (range `split` covers steps_per_split 64-token steps and goes to out + split * split_stride).
template <int NS>
__device__ __forceinline__ void wgrad_dma_tile(const bf16* __restrict__ G, int64_t ldg,
                                               const bf16* __restrict__ A, int64_t lda,
                                               int M, int N, int K, int steps_per_split,
                                               float* __restrict__ out, int64_t split_stride, int tile, int split) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // scalar: M0 values need no lane read-out
    const int wp = wave >> 1, wq = wave & 1;                       // 2 x 2 wavefronts, 64 x 64 each
    const int tiles_q = (K + WD_BQ - 1) / WD_BQ;
    const int tiles = ((N + WD_BP - 1) / WD_BP) * tiles_q;
    // The slow tile index is the one along the WIDER output dimension.
    const int tiles_p = tiles / tiles_q;
    int tp, tq;
    if (K > N) { tq = tile / tiles_p; tp = tile - tq * tiles_p; }
    else { tp = tile / tiles_q; tq = tile - tp * tiles_q; }
    const int p0 = tp * WD_BP, q0 = tq * WD_BQ;
    const int total_steps = (M + WD_BR - 1) / WD_BR;
    const int step0 = split * steps_per_split;
    const int nsteps = max(0, min(steps_per_split, total_steps - step0));

    // Each operand tile is 16 wavefront-wide loads of 4 token rows; wavefront w issues loads
    // w, w+4, w+8, w+12 of G and the same of A.  Lane l: row 4*i + l/16, LDS position l%16.
    constexpr int LPW = 8;
    int rowl[4], chunk[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int i = wave + 4 * t;
        rowl[t] = 4 * i + (lane >> 4);
        chunk[t] = (lane & 15) ^ (4 * (rowl[t] & 3));
    }
    const bf16* zero = reinterpret_cast<const bf16*>(g_zero_chunk);
    auto issue = [&](int st, int stage) {
        const int mbase = (step0 + st) * WD_BR;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int m = mbase + rowl[t];
            const int gp = p0 + chunk[t] * 8, gq = q0 + chunk[t] * 8;
            const bf16* sg = (m < M && gp < N) ? G + (int64_t)m * ldg + gp : zero;
            const bf16* sa = (m < M && gq < K) ? A + (int64_t)m * lda + gq : zero;
            const int i = wave + 4 * t;
            __builtin_amdgcn_global_load_lds(GLB_PTR(sg), LDS_PTR(void, smem + stage * WD_STAGE + i * 1024), 16, 0, 0);
            __builtin_amdgcn_global_load_lds(GLB_PTR(sa), LDS_PTR(void, smem + stage * WD_STAGE + WD_TILE + i * 1024), 16, 0, 0);
        }
    };

    f32x16_t acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

#pragma unroll
    for (int s = 0; s < NS - 1; ++s)
        if (s < nsteps) issue(s, s);

    if constexpr (NS == 2) {
        // Hand-placed fragment reads (see mfma.h): one step ahead, every product group waits only
        // for its own 8 transpose reads.  Stage parity and "is there a next stage" are compile-time
        // tags so that the loop body has no branch.
        const unsigned lds0 = (unsigned)(uintptr_t)LDS_PTR(unsigned char, smem);
        unsigned g_addr[2], a_addr[2];
        {
            const int jj = lane & 15, q = lane >> 4;
            const int r = (q >> 1) * 8 + (jj >> 2);
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int cg = wp * 64 + i * 32 + (q & 1) * 16 + 4 * (jj & 3);
                const int ca = wq * 64 + i * 32 + (q & 1) * 16 + 4 * (jj & 3);
                g_addr[i] = lds0 + r * 256 + (((cg >> 3) ^ (4 * (r & 3))) * 16) + (cg & 7) * 2;
                a_addr[i] = lds0 + WD_TILE + r * 256 + (((ca >> 3) ^ (4 * (r & 3))) * 16) + (ca & 7) * 2;
            }
        }
        // Full steps (all 64 token rows inside M) are loaded in the scalar-base form: per-lane 32-bit
        // offsets fixed for the whole kernel, the scalar base advancing by 64 rows per step; tile
        // columns beyond N / K re-read the last valid 8 (those outputs are never stored).  Only a
        // ragged last step needs the zero-filling form above.
        unsigned voff_g[4], voff_a[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            voff_g[t] = (unsigned)(rowl[t] * ldg * 2 + min(chunk[t] * 8, N - 8 - p0) * 2);
            voff_a[t] = (unsigned)(rowl[t] * lda * 2 + min(chunk[t] * 8, K - 8 - q0) * 2);
        }
        const char* g_base = reinterpret_cast<const char*>(G + p0);
        const char* a_base = reinterpret_cast<const char*>(A + q0);
        auto issue_fast = [&](int st, int stage) {
            const int64_t mbase = (int64_t)(step0 + st) * WD_BR;
            const char* gs = g_base + mbase * ldg * 2;
            const char* as = a_base + mbase * lda * 2;
            const unsigned sb = lds0 + stage * WD_STAGE;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int i = wave + 4 * t;
                dma16_sbase(gs, voff_g[t], sb + i * 1024);
                dma16_sbase(as, voff_a[t], sb + WD_TILE + i * 1024);
            }
        };
        auto issue_any = [&](int st, int stage) {
            if ((step0 + st + 1) * WD_BR <= M) issue_fast(st, stage);
            else issue(st, stage);
        };
        auto body = [&](auto stage_tag, auto next_tag, int st) {
            constexpr int SOFF = decltype(stage_tag)::value * WD_STAGE;
            constexpr bool has_next = decltype(next_tag)::value;
            __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));
            __builtin_amdgcn_s_barrier();
            u32x4_t a[4][2], b[4][2];
            auto read_group = [&](auto kk_tag) {
                constexpr int kk = decltype(kk_tag)::value;
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    a[kk][i] = join64(lds_read_tr16_b64(g_addr[i], SOFF + kk * 16 * 256),
                                      lds_read_tr16_b64(g_addr[i], SOFF + kk * 16 * 256 + 4 * 256));
                    b[kk][i] = join64(lds_read_tr16_b64(a_addr[i], SOFF + kk * 16 * 256),
                                      lds_read_tr16_b64(a_addr[i], SOFF + kk * 16 * 256 + 4 * 256));
                }
            };
            auto products = [&](int kk) {
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j) acc[i][j] = mfma32(as_bf16x8(a[kk][i]), as_bf16x8(b[kk][j]), acc[i][j]);
                __builtin_amdgcn_sched_barrier(0);
            };
            using I0 = std::integral_constant<int, 0>; using I1 = std::integral_constant<int, 1>;
            using I2 = std::integral_constant<int, 2>; using I3 = std::integral_constant<int, 3>;
            read_group(I0{}); read_group(I1{});
            if (has_next) issue_any(st + 1, 1 - decltype(stage_tag)::value);
            lds_wait4<8>(a[0][0], a[0][1], b[0][0], b[0][1]); products(0);
            read_group(I2{});
            lds_wait4<8>(a[1][0], a[1][1], b[1][0], b[1][1]); products(1);
            read_group(I3{});
            lds_wait4<8>(a[2][0], a[2][1], b[2][0], b[2][1]); products(2);
            lds_wait4<0>(a[3][0], a[3][1], b[3][0], b[3][1]); products(3);
        };
        using S0 = std::integral_constant<int, 0>; using S1 = std::integral_constant<int, 1>;
        int st = 0;
        for (; st + 2 < nsteps; st += 2) {
            body(S0{}, std::true_type{}, st);
            body(S1{}, std::true_type{}, st + 1);
        }
        if (st + 2 == nsteps) {
            body(S0{}, std::true_type{}, st);
            body(S1{}, std::false_type{}, st + 1);
        } else if (st + 1 == nsteps) {
            body(S0{}, std::false_type{}, st);
        }
    } else
    for (int st = 0; st < nsteps; ++st) {
        if (st + NS - 2 < nsteps) __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0((NS - 2) * LPW));
        else __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));
        __builtin_amdgcn_s_barrier();
        if (st + NS - 1 < nsteps) issue(st + NS - 1, (st + NS - 1) % NS);
        const unsigned char* Gt = smem + (st % NS) * WD_STAGE;
        const unsigned char* At = Gt + WD_TILE;
#pragma unroll
        for (int kk = 0; kk < WD_BR / 16; ++kk) {
            bf16x8_t a[2], b[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) a[i] = tr_frag_swz(Gt, kk * 16, wp * 64 + i * 32, lane);
#pragma unroll
            for (int j = 0; j < 2; ++j) b[j] = tr_frag_swz(At, kk * 16, wq * 64 + j * 32, lane);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[i][j] = mfma32(a[i], b[j], acc[i][j]);
        }
    }

    float* o = out + (int64_t)split * split_stride;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int q = q0 + wq * 64 + j * 32 + (lane & 31);
        if (q >= K) continue;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int pb = p0 + wp * 64 + i * 32 + 4 * (lane >> 5);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int p = pb + 8 * (v >> 2) + (v & 3);
                if (p < N) o[(int64_t)p * K + q] = acc[i][j][v];
            }
        }
    }
}

// Each XCD takes one contiguous run of the (token range, tile) order, token range slowest: an XCD
// then works on one or two token ranges and on a block of tiles inside them, so both operands are
// partitioned over the XCDs' L2s (with every XCD walking all ranges of its tiles, each of them read
// the whole of one operand).
template <int NS>
__global__ __launch_bounds__(256) void wgrad_dma_kernel(const bf16* __restrict__ G, int64_t ldg,
                                                        const bf16* __restrict__ A, int64_t lda,
                                                        int M, int N, int K, int steps_per_split,
                                                        float* __restrict__ out, int64_t split_stride) {
    const int tiles = ((N + WD_BP - 1) / WD_BP) * ((K + WD_BQ - 1) / WD_BQ);
    const int lin = xcd_remap(blockIdx.x, gridDim.x);
    const int split = lin / tiles;
    wgrad_dma_tile<NS>(G, ldg, A, lda, M, N, K, steps_per_split, out, split_stride, lin - split * tiles, split);
}

// Several weight gradients over the same M tokens in one launch (the four of a transformer block): the tiles of all
// of them form one list, so that together they fill the device where each alone would have to cut its token range
// into pieces (and sum the pieces afterwards) to do so.
template <int NS>
__global__ __launch_bounds__(256) void wgrad_dma_group_kernel(WgradGroup grp, int M, int steps_per_split) {
    const int lin = xcd_remap(blockIdx.x, gridDim.x);
    const int split = lin / grp.tiles_total;
    const int gt = lin - split * grp.tiles_total;
    int pi = 0;
#pragma unroll
    for (int k = 1; k < WGRAD_GROUP_MAX; ++k)
        if (k < grp.count && gt >= grp.p[k].tile0) pi = k;
    const WgradProblem& q = grp.p[pi];
    wgrad_dma_tile<NS>(q.G, q.ldg, q.A, q.lda, M, q.N, q.K, steps_per_split, q.out, q.split_stride, gt - q.tile0, split);
}

int launch_wgrad_dma_group(hipStream_t s, WgradGroup grp, int M, int S, int sps) {
    static LdsLimit lim;
    if (int rc = lim.ensure(reinterpret_cast<const void*>(wgrad_dma_group_kernel<2>), 2 * WD_STAGE)) return rc;
    hipLaunchKernelGGL(wgrad_dma_group_kernel<2>, dim3(grp.tiles_total * S), dim3(256), 2 * WD_STAGE, s, grp, M, sps);
    REV_HIP(hipGetLastError());
    return REV_OK;
}

int launch_wgrad_dma(hipStream_t s, const bf16* G, int64_t ldg, const bf16* A, int64_t lda, int M, int N, int K,
                     int S, int sps, float* out) {
    const int tiles = ((N + WD_BP - 1) / WD_BP) * ((K + WD_BQ - 1) / WD_BQ);
    static LdsLimit lim;
    if (int rc = lim.ensure(reinterpret_cast<const void*>(wgrad_dma_kernel<2>), 2 * WD_STAGE)) return rc;
    hipLaunchKernelGGL(wgrad_dma_kernel<2>, dim3(tiles * S), dim3(256), 2 * WD_STAGE, s, G, ldg, A, lda, M, N, K, sps, out, (int64_t)N * K);
    REV_HIP(hipGetLastError());
    return REV_OK;
}

}  // namespace rev
