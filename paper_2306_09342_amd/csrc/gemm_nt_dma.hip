// NT GEMM, pipelined flavour:  C[M,N] (+epilogue) = A[M,K] * B[N,K]^T  for K % 32 == 0 (64-wide stages
// when K % 64 == 0, the tuned case).
//
// Operand tiles travel HBM -> LDS with the direct-to-LDS loads of gfx950
// (global_load_lds_dwordx4): no staging registers, no LDS store instructions.
// A ring of NS stages is kept in flight; a stage is consumed after
// s_waitcnt vmcnt(.) (this wavefront's loads of the stage have landed) and one
// workgroup barrier (everybody's have, and everybody is done reading the stage
// that is about to be refilled).
//
// LDS tile layout: rows of 64 bf16 (128 B), dense.  A direct-to-LDS load drops the
// 64 lanes' 16-byte pieces contiguously, so instead of padding the rows the
// 16-byte chunk c of row r is kept at position c ^ ((r >> 1) & 7): each lane
// simply fetches the global chunk that belongs at its LDS position.  Fragment
// reads (16 rows x one chunk per quarter-wavefront) then hit 16 distinct bank
// groups.
//
// The matrix-core product is taken as C^T = B * A^T (weights on the A port), so a
// lane's accumulator quad holds 4 consecutive output columns; the tile goes
// through LDS once and leaves in full contiguous rows with 16-byte accesses,
// the epilogue (bias, GELU, GELU', residual) applied on the way out.
//
// Three tile shapes run the tuned loop: 128x128 with four wavefronts of 64x64 (two
// workgroups per CU, the general case); 160x128 with two wavefronts of 160x64
// (7 fragment reads per 10 products, one wavefront per SIMD), which a launch that
// has the device to itself picks when 128-row tiles would leave a short, ragged
// last round of workgroups; and 64x128 with two wavefronts of 64x64 for launches
// too small to give every second CU a 128-row tile.
#include "gemm_epilogue.h"
#include <type_traits>

namespace rev {

template <int BM, int BN, int WM, int WN, int BK, int NS, int KIND, bool BKM>
__global__ __launch_bounds__(WM * WN * 64) void gemm_nt_dma_kernel(const bf16* __restrict__ A, int64_t lda,
                                                                    const bf16* __restrict__ B, int64_t ldb,
                                                                    int M, int N, int K, Epi epi, int gn) {
    constexpr int NW = WM * WN;
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    constexpr int ROWB = BK * 2;                         // bytes per tile row
    constexpr int CPR = BK / 8;                          // 16-byte chunks per row (8 or 4)
    constexpr int RPI = 64 / CPR;                        // rows covered by one wavefront-wide load
    // B is either [N, K] (rows contraction-contiguous, like A) or, with BKM, [K, N]: then its tile
    // is BK rows of BN columns, kept as it lies in memory and read with the LDS transpose read
    static_assert(!BKM || BN == 128, "K-major B tiles have 256-byte rows");
    constexpr int A_BYTES = BM * ROWB, B_BYTES = BN * ROWB, STAGE = A_BYTES + B_BYTES;
    constexpr int IA = BM / RPI, IB = B_BYTES / 1024;    // wavefront-wide loads per stage
    constexpr int LPW = (IA + IB) / NW;                  // ... per wavefront
    static_assert(BK == 64 || BK == 32, "BK");
    static_assert(IA % NW == 0 && IB % NW == 0, "loads must split evenly over the wavefronts");
    static_assert(NS == 1 || (NS - 2) * LPW < 64, "vmcnt range");
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    // the wavefront index as a scalar: LDS destinations of the direct-to-LDS loads (M0) then need no
    // per-load lane read-out
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int g = lane >> 5;
    // Tile order: column groups of `gn` n-tiles, each group walked over all m-tiles, n fastest inside
    // a group; every XCD gets one contiguous run of that order.  The weight slice of a group
    // (gn * BN rows of B) then stays in the XCD's L2 while the activation panels stream past it.
    const int tiles_n = (N + BN - 1) / BN, tiles_m = (M + BM - 1) / BM;
    const int tile = xcd_remap(blockIdx.x, gridDim.x);
    const int per_group = gn * tiles_m;
    const int grp = tile / per_group, in_grp = tile - grp * per_group;
    const int gw = min(gn, tiles_n - grp * gn);              // width of this (possibly last, narrower) group
    const int m0 = (in_grp / gw) * BM, n0 = (grp * gn + in_grp % gw) * BN;

    // chunk c of row r is kept at position c ^ swz(r): 16 consecutive rows x one chunk -> 16 distinct bank groups
    auto swz = [](int r) { return BK == 64 ? ((r >> 1) & 7) : ((r >> 2) & 3); };

    // Sources of this wavefront's loads: a scalar base per operand (the tile's first row / column,
    // advanced along K per stage) plus a 32-bit per-lane byte offset inside the tile's panel, which
    // is what the scalar-base addressing form of the load takes: no 64-bit vector adds per load.
    // Rows beyond M or N re-read the last valid row; K-major B columns beyond N re-read the last
    // valid 8 columns (such output rows / columns are never stored).
    unsigned voff[LPW];
    int dst[LPW];
#pragma unroll
    for (int t = 0; t < LPW; ++t) {
        const int i = wave + NW * t;                     // load index within the stage: A first, then B
        const bool isA = (NW * t) < IA;                  // uniform per t because IA % NW == 0
        const int ii = isA ? i : i - IA;
        const int row = ii * RPI + lane / CPR;
        const int chunk = (lane % CPR) ^ swz(row);
        if (isA) {
            voff[t] = (unsigned)(min(row, M - 1 - m0) * lda * 2 + chunk * 16);
            dst[t] = ii * 1024;
        } else if (!BKM) {
            voff[t] = (unsigned)(min(row, N - 1 - n0) * ldb * 2 + chunk * 16);
            dst[t] = A_BYTES + ii * 1024;
        } else {
            // 4 contraction rows of 16 chunks per load; chunk c of row r at position c ^ (4 * (r & 3))
            const int krow = ii * 4 + (lane >> 4);
            const int col = min(((lane & 15) ^ (4 * (krow & 3))) * 8, N - 8 - n0);
            voff[t] = (unsigned)(krow * ldb * 2 + col * 2);
            dst[t] = A_BYTES + ii * 1024;
        }
    }
    const char* a_base = reinterpret_cast<const char*>(A + (int64_t)m0 * lda);
    const char* b_base = reinterpret_cast<const char*>(BKM ? B + n0 : B + (int64_t)n0 * ldb);
    const int64_t bstep = BKM ? (int64_t)BK * ldb * 2 : (int64_t)BK * 2;       // B advance per stage, bytes
    // loads t0 <= t < t1 of the stage (the whole stage: 0, LPW)
    auto issue_part = [&](int kt, int stage, int t0, int t1) {
        const char* ak = a_base + (int64_t)kt * (BK * 2);
        const char* bk = b_base + kt * bstep;
#pragma unroll
        for (int t = 0; t < LPW; ++t) {
            if (t < t0 || t >= t1) continue;
            const bool isA = (NW * t) < IA;
            const char* p = (isA ? ak : bk) + voff[t];
            __builtin_amdgcn_global_load_lds(GLB_PTR(p), LDS_PTR(void, smem + stage * STAGE + dst[t]), 16, 0, 0);
        }
    };
    auto issue = [&](int kt, int stage) { issue_part(kt, stage, 0, LPW); };
    // With one wavefront per SIMD the loads of the next stage are handed out in slices between the
    // product groups of the current one, so the matrix cores start right after the barrier.
    constexpr bool SPREAD = (NW == 4 && TM * TN >= 16 && NS == 2 && LPW % (BK / 16) == 0);
    // 64x64 per wavefront (four wavefronts, the default 128x128 tile) or 160x64 (two wavefronts, the tall tile)
    constexpr bool HANDPLACED_SHAPE = (((TM == 2 && (NW == 4 || NW == 2)) || (TM == 5 && NW == 2)) && TN == 2 && BK == 64 && NS == 2 && !SPREAD);

    // Epilogue geometry (a wavefront's 32-row panels leave through LDS in full rows) and, for the
    // epilogues that read a second operand (residual stream, saved pre-activation), that operand:
    // it does not depend on the products, so it is requested before the main loop and has landed
    // long before it is needed.
    constexpr int CW = TN * 32, CP = CW + 4;
    constexpr int LPR = CW / 4;                           // lanes per row
    constexpr int RPP = 64 / LPR;                         // rows per pass
    constexpr int NP = 32 / RPP;
    const int c4 = lane % LPR, rr = lane / LPR;
    const int n = n0 + wn * CW + 4 * c4;
    // (float32 residual rows cost 4 registers each: only the first panel's are held across the main
    // loop, the second panel's are requested when the epilogue starts)
    constexpr int PRE = !HANDPLACED_SHAPE ? 0 : (KIND == EPI_GELU_BWD ? (TM > 2 ? 2 : TM) : (KIND == EPI_RESIDUAL ? 1 : 0));
    f32x4_t opnd_pre[TM][NP];
    if (PRE > 0 && n < N) {
#pragma unroll
        for (int i = 0; i < PRE; ++i)
#pragma unroll
            for (int p = 0; p < NP; ++p)
                opnd_pre[i][p] = epi_load4<KIND>(epi, min(m0 + wm * TM * 32 + i * 32 + rr + p * RPP, M - 1), n);
    }

    f32x16_t acc[TN][TM];
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[j][i][v] = 0.f;

    const int nk = K / BK;
#pragma unroll
    for (int s = 0; s < NS - 1; ++s)
        if (s < nk) issue(s, s);

    // fragment addressing: row r of a tile region, chunk (2*kk + g) swizzled
    const int fr = lane & 31;
    int koff[BK / 16];
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) koff[kk] = ((2 * kk + g) ^ swz(fr)) << 4;
    const int a_row = (wm * TM * 32 + fr) * ROWB;
    const int b_row = A_BYTES + (wn * TN * 32 + fr) * ROWB;

    // The default shape (128x128x64 tile, 64x64 per wavefront, 2 stages) and the tall one (160x128x64, 160x64 per
    // wavefront) take the hand-placed path.
    constexpr bool HANDPLACED = HANDPLACED_SHAPE;
    if constexpr (HANDPLACED) {
        const unsigned lds0 = (unsigned)(uintptr_t)LDS_PTR(unsigned char, smem);
        unsigned a_addr[4], b_addr[4];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            a_addr[kk] = lds0 + a_row + koff[kk];
            b_addr[kk] = lds0 + b_row + koff[kk];
        }
        // K-major B: base addresses of the two 32-column fragments of this wavefront (step 0, low half)
        unsigned bt_addr[2] = {0, 0};
        if (BKM) {
            const int jj = lane & 15, q = lane >> 4;
            const int r = (q >> 1) * 8 + (jj >> 2);
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int c = wn * 64 + j * 32 + (q & 1) * 16 + 4 * (jj & 3);
                const int pos = (c >> 3) ^ (4 * (r & 3));
                bt_addr[j] = lds0 + A_BYTES + r * 256 + pos * 16 + (c & 7) * 2;
            }
        }
        // has_next is a compile-time tag: a branch around the loads inside the loop body makes the
        // register allocator shuttle all 64 accumulators between register files every iteration
        // this path issues its global loads in the scalar-base form
        auto issue = [&](int kt, int stage) {
            const char* ak = a_base + (int64_t)kt * (BK * 2);
            const char* bk = b_base + kt * bstep;
            const unsigned sbase = lds0 + stage * STAGE;
#pragma unroll
            for (int t = 0; t < LPW; ++t)
                dma16_sbase((NW * t) < IA ? ak : bk, voff[t], sbase + dst[t]);
        };
        auto stage_body = [&](auto stage_tag, auto next_tag, int kt) {
            // the stage offset rides in the instruction's 16-bit offset field
            constexpr int SOFF = decltype(stage_tag)::value * STAGE;
            static_assert(SOFF + (TM - 1) * 32 * ROWB < 65536 && SOFF + 3 * 16 * 256 + 4 * 256 < 65536, "LDS read offsets are 16 bits wide");
            constexpr bool has_next = decltype(next_tag)::value;
            __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));
            __builtin_amdgcn_s_barrier();
            u32x4_t a[4][TM], b[4][2];
            auto read_group = [&](auto kk_tag) {
                constexpr int kk = decltype(kk_tag)::value;
                a[kk][0] = lds_read_b128(a_addr[kk], SOFF);
                a[kk][1] = lds_read_b128(a_addr[kk], SOFF + 32 * ROWB);
                if constexpr (TM == 5) {
                    a[kk][2] = lds_read_b128(a_addr[kk], SOFF + 64 * ROWB);
                    a[kk][3] = lds_read_b128(a_addr[kk], SOFF + 96 * ROWB);
                    a[kk][4] = lds_read_b128(a_addr[kk], SOFF + 128 * ROWB);
                }
                if (BKM) {
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        b[kk][j] = join64(lds_read_tr16_b64(bt_addr[j], SOFF + kk * 16 * 256),
                                          lds_read_tr16_b64(bt_addr[j], SOFF + kk * 16 * 256 + 4 * 256));
                } else {
                    b[kk][0] = lds_read_b128(b_addr[kk], SOFF);
                    b[kk][1] = lds_read_b128(b_addr[kk], SOFF + 32 * ROWB);
                }
            };
            auto products = [&](int kk) {
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int i = 0; i < TM; ++i) acc[j][i] = mfma32(as_bf16x8(b[kk][j]), as_bf16x8(a[kk][i]), acc[j][i]);
                __builtin_amdgcn_sched_barrier(0);       // the products stay between their wait and the next one
            };
            // waits until at most N younger LDS reads are outstanding; carries step kk's fragments
            auto wait_group = [&](auto n_tag, int kk) {
                constexpr int N = decltype(n_tag)::value;
                if constexpr (TM == 5) lds_wait7<N>(a[kk][0], a[kk][1], a[kk][2], a[kk][3], a[kk][4], b[kk][0], b[kk][1]);
                else lds_wait4<N>(a[kk][0], a[kk][1], b[kk][0], b[kk][1]);
            };
            using I0 = std::integral_constant<int, 0>; using I1 = std::integral_constant<int, 1>;
            using I2 = std::integral_constant<int, 2>; using I3 = std::integral_constant<int, 3>;
            constexpr int RPK = TM + (BKM ? 4 : 2);       // LDS reads per step
            using NRPK = std::integral_constant<int, RPK>; using N0 = std::integral_constant<int, 0>;
            // one step ahead, as the compiler would order it, but every product group waits only for
            // its own operands (the reads of the step after it stay in flight)
            read_group(I0{}); read_group(I1{});
            if (has_next) issue(kt + 1, 1 - decltype(stage_tag)::value);
            wait_group(NRPK{}, 0); read_group(I2{}); products(0);
            wait_group(NRPK{}, 1); read_group(I3{}); products(1);
            wait_group(NRPK{}, 2); products(2);
            wait_group(N0{}, 3);   products(3);
        };
        using S0 = std::integral_constant<int, 0>; using S1 = std::integral_constant<int, 1>;
        int kt = 0;
        for (; kt + 2 < nk; kt += 2) {
            stage_body(S0{}, std::true_type{}, kt);
            stage_body(S1{}, std::true_type{}, kt + 1);
        }
        if (kt + 2 == nk) {
            stage_body(S0{}, std::true_type{}, kt);
            stage_body(S1{}, std::false_type{}, kt + 1);
        } else {
            stage_body(S0{}, std::false_type{}, kt);
        }
    } else
    for (int kt = 0; kt < nk; ++kt) {
        if (NS == 1) {
            // single buffer: latency is hidden by the other workgroups resident on the CU
            __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));
            __builtin_amdgcn_s_barrier();                 // everybody is done reading the buffer
            issue(kt, 0);
            __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));
            __builtin_amdgcn_s_barrier();
        } else {
            // loads of stage kt are older than the (NS-2) stages issued after them
            if (kt + NS - 2 < nk) __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(NS > 1 ? (NS - 2) * LPW : 0));
            else __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));
            __builtin_amdgcn_s_barrier();
            if (!SPREAD && kt + NS - 1 < nk) issue(kt + NS - 1, (kt + NS - 1) % NS);
        }
        const unsigned char* st = smem + (kt % NS) * STAGE;
        // fragments of step kk+1 are requested before the products of step kk are issued
        bf16x8_t a[2][TM], b[2][TN];
        auto load_frags = [&](int kk, int slot) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
                a[slot][i] = *reinterpret_cast<const bf16x8_t*>(st + a_row + i * 32 * ROWB + koff[kk]);
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                if (BKM) b[slot][j] = tr_frag_swz(st + A_BYTES, kk * 16, wn * TN * 32 + j * 32, lane);
                else b[slot][j] = *reinterpret_cast<const bf16x8_t*>(st + b_row + j * 32 * ROWB + koff[kk]);
            }
        };
        load_frags(0, 0);
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            if (kk + 1 < BK / 16) load_frags(kk + 1, (kk + 1) & 1);
            if (SPREAD && kt + 1 < nk) {
                constexpr int PER = LPW / (BK / 16);
                issue_part(kt + 1, (kt + 1) % NS, kk * PER, (kk + 1) * PER);
            }
            __builtin_amdgcn_sched_barrier(0);       // keep the LDS reads ahead of the products that hide them
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int i = 0; i < TM; ++i) acc[j][i] = mfma32(b[kk & 1][j], a[kk & 1][i], acc[j][i]);
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    // ---- epilogue through LDS, 32 rows at a time: wavefront-private [32][TN*32 + 4] float32 ----
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));
    __builtin_amdgcn_s_barrier();                         // every wavefront is done with the operand stages
    float* ct = reinterpret_cast<float*>(smem) + wave * (32 * CP);
    if ((KIND == EPI_RESIDUAL || KIND == EPI_GELU_BWD) && n < N) {
#pragma unroll
        for (int i = PRE; i < TM; ++i)
#pragma unroll
            for (int p = 0; p < NP; ++p)
                opnd_pre[i][p] = epi_load4<KIND>(epi, min(m0 + wm * TM * 32 + i * 32 + rr + p * RPP, M - 1), n);
    }
    f32x4_t csum = {0.f, 0.f, 0.f, 0.f};
    f32x4_t bv = {0.f, 0.f, 0.f, 0.f};                    // this lane's 4 columns never change: one bias load
    if ((KIND == EPI_BIAS || KIND == EPI_BIAS_GELU || KIND == EPI_RESIDUAL) && n < N)
        bv = ld_bf16x4(reinterpret_cast<const bf16*>(epi.bias) + n);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                f32x4_t v = {acc[j][i][4 * vq], acc[j][i][4 * vq + 1], acc[j][i][4 * vq + 2], acc[j][i][4 * vq + 3]};
                *reinterpret_cast<f32x4_t*>(ct + fr * CP + j * 32 + 8 * vq + 4 * g) = v;
            }
        // the region is private to the wavefront and LDS operations of a wavefront complete in order
        // first every LDS read and every epilogue operand load of the 32-row panel, then the
        // arithmetic and the stores: one memory round trip per panel instead of one per row group
        f32x4_t v[NP], opnd[NP];
        const int mrow = m0 + wm * TM * 32 + i * 32 + rr;
#pragma unroll
        for (int p = 0; p < NP; ++p) v[p] = *reinterpret_cast<const f32x4_t*>(ct + (p * RPP + rr) * CP + 4 * c4);
        if (n < N) {
#pragma unroll
            for (int p = 0; p < NP; ++p) opnd[p] = opnd_pre[i][p];
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                const int m = mrow + p * RPP;
                if (m < M) {
                    const f32x4_t o = epi_store4<KIND>(epi, m, n, v[p], bv, opnd[p]);
                    if (KIND == EPI_GELU_BWD) csum += o;
                }
            }
        }
    }
    // fused bias gradient: column sums of this wavefront's 64-row strip, lanes folded in a fixed order
    if (KIND == EPI_GELU_BWD && TM * 32 == 64 && epi.colsum != nullptr) {   // strips are 64 rows
#pragma unroll
        for (int off = LPR; off < 64; off <<= 1)
#pragma unroll
            for (int k = 0; k < 4; ++k) csum[k] += __shfl_xor(csum[k], off, 64);
        if (rr == 0 && n < N) {
            const int strip = (m0 + wm * TM * 32) >> 6;
            *reinterpret_cast<f32x4_t*>(epi.colsum + (int64_t)strip * N + n) = csum;
        }
    }
}

template <int BM, int BN, int WM, int WN, int BK, int NS, int KIND, bool BKM>
static int launch_dma(hipStream_t s, const bf16* A, int64_t lda, const bf16* B, int64_t ldb, int M, int N, int K,
                      const Epi& epi) {
    constexpr int NW = WM * WN;
    constexpr size_t stage_bytes = (size_t)NS * (BM + BN) * BK * 2;
    constexpr size_t epi_bytes = (size_t)NW * 32 * (BN / WN + 4) * 4;
    constexpr size_t shmem = stage_bytes > epi_bytes ? stage_bytes : epi_bytes;
    static LdsLimit lim;
    auto kern = gemm_nt_dma_kernel<BM, BN, WM, WN, BK, NS, KIND, BKM>;
    if (int rc = lim.ensure(reinterpret_cast<const void*>(kern), (int)shmem)) return rc;
    const int tiles_n = (N + BN - 1) / BN;
    const int tiles = ((M + BM - 1) / BM) * tiles_n;
    // Group width.  An XCD runs about 64 tiles at a time; with at most 8 n-tiles per group it holds 8 or
    // more m-rows of the group at once, all sweeping the same k-slices of the same slice of B, which
    // therefore stays in L2 (measured: L2 misses of the 24-n-tile GEMMs halve).  Narrow outputs
    // (up to 12 n-tiles) are left ungrouped: re-reading A once per group would cost more than it saves.
    const int gn = tiles_n <= 12 ? tiles_n : 8;
    hipLaunchKernelGGL(kern, dim3(tiles), dim3(NW * 64), shmem, s, A, lda, B, ldb, M, N, K, epi, gn);
    REV_HIP(hipGetLastError());
    return REV_OK;
}

// number of 64-row strips whose column sums the EPI_GELU_BWD epilogue writes (whole tiles, so every
// strip of every launched workgroup is written, those past M with zeros)
int gemm_colsum_strips(int M) {
    return ((M + 127) / 128) * 2;
}

// Cost of a launch in units of "one tile per workgroup slot": the chip holds 512 workgroups of either
// shape (two per CU); a last round that leaves at most one workgroup per CU was measured at about 0.55
// of a full round, any fuller one costs a whole round.
static double rounds_cost(int tiles) {
    const int full = tiles / 512, rem = tiles % 512;
    return full + (rem == 0 ? 0.0 : (rem <= 256 ? 0.55 : 1.0));
}
// 160x128 tiles do 1.25x the work of 128x128 ones at about 0.9 of their rate.  Only launches with more than
// one full round of 128-row tiles are considered: below that the chip is not full and the cost of a
// partly filled round does not follow the model (measured: the tall tile loses there).
static bool tall_tiles_pay(int M, int N) {
    const int tn = (N + 127) / 128;
    if (((M + 127) / 128) * tn <= 512) return false;
    const double c128 = rounds_cost(((M + 127) / 128) * tn) * 128.0;
    const double c160 = rounds_cost(((M + 159) / 160) * tn) * 160.0 * 1.10;
    return c160 < 0.97 * c128;
}

template <int KIND, bool BKM>
static int dispatch_dma(hipStream_t s, const bf16* A, int64_t lda, const bf16* B, int64_t ldb, int M, int N, int K,
                        const Epi& epi) {
    // K a multiple of 32 but not of 64 (e.g. width 96): the same tile with 32-wide stages
    if (K % 64 != 0) return launch_dma<128, 128, 2, 2, 32, 2, KIND, BKM>(s, A, lda, B, ldb, M, N, K, epi);
    // Small launches (at most one 128-row tile for every second CU): 64x128 tiles run by two
    // wavefronts of 64x64 put twice as many workgroups on the chip (8-13 % faster at 197...1576 rows).
    // Never with fused column sums (their strips belong to 128-row tiles).
    if (epi.colsum == nullptr && ((M + 127) / 128) * ((N + 127) / 128) <= 128)
        return launch_dma<64, 128, 1, 2, 64, 2, KIND, BKM>(s, A, lda, B, ldb, M, N, K, epi);
    // 160-row tiles (two wavefronts of 160x64) when they turn a short ragged second round of
    // 128-row tiles into a single round.  Only for launches that have the device to themselves:
    // next to another stream's kernels that round is filled anyway and the larger LDS footprint
    // keeps the neighbour out (measured: sequential schedule faster, parallel schedule 5 % slower).
    // Each output element sums the same products in the same order under every shape, so the choice
    // does not change a bit of the result.
    if (epi.solo && epi.colsum == nullptr && tall_tiles_pay(M, N))
        return launch_dma<160, 128, 1, 2, 64, 2, KIND, BKM>(s, A, lda, B, ldb, M, N, K, epi);
    return launch_dma<128, 128, 2, 2, 64, 2, KIND, BKM>(s, A, lda, B, ldb, M, N, K, epi);
}

// Pipelined path; the caller has checked K % 32 == 0, N % 8 == 0 and 16-byte alignment of every row.
// b_kmajor = false: B is [N, K];  true: B is [K, N] (C = A * B).
int gemm_bf16_dma(hipStream_t s, const bf16* A, int64_t lda, const bf16* B, int64_t ldb,
                  int M, int N, int K, const Epi& epi, bool b_kmajor) {
    switch (epi.kind) {
#define CASE(KIND) case KIND: return b_kmajor ? dispatch_dma<KIND, true>(s, A, lda, B, ldb, M, N, K, epi) \
                                              : dispatch_dma<KIND, false>(s, A, lda, B, ldb, M, N, K, epi);
        CASE(EPI_BIAS) CASE(EPI_BIAS_GELU) CASE(EPI_RESIDUAL) CASE(EPI_GELU_BWD) CASE(EPI_PLAIN) CASE(EPI_PLAIN_F32)
#undef CASE
    }
    set_error("gemm_bf16: unknown epilogue");
    return REV_EINVAL;
}

}  // namespace rev
