// Stage transition of a hierarchical reversible model (paper Sec. 3.4, "downsample block"): the two
// residual streams are fused (by averaging, or by a small MLP), every 2x2 neighbourhood of the token grid
// is concatenated (C -> 4C features), normalised by a LayerNorm and reduced by a bias-free linear map to 2C.
// The block is not reversible: its backward pass gets the block's inputs from the caller.
//
// Forward:   z0 = (X1 + X2) / 2                                     (fusion by averaging), or
//            z0 = gelu([X1 | X2] * Wa^T + ba) * Wb^T + bb           (fusion by a small MLP, Wa [C, 2C], Wb [C, C])
//            z[o, q*C + c] = z0[src(o,q), c],  q = 2*dy + dx;   n = LN(z),  out = n * W^T
// Backward:  dout = dOutA + dOutB (both streams of the next stage start from `out`)
//            dW = dout^T * n,  dn = dout * W,  dz = LNbwd(dn),  dz0[src] = dz,
//            averaging: dX1 = dX2 = dz0 / 2;   MLP: the two linear maps and the GELU backwards, recomputed
//            from X1, X2 (the block keeps nothing between its two calls)
//
// Tokens are stored window by window (the windows are the attention sequences of the stages), on
// both sides of the block.  The gather, the average and the LayerNorm are one kernel (a wavefront
// per output row, the row in registers); its backward is one kernel too, which recomputes the
// gathered row, applies the LayerNorm backward and scatters the halves to both streams.  The three
// contractions are the library's GEMM kernels.
#include "common.h"
#include "rowwise.h"

namespace rev {

struct MergeGeom {
    int B, Gh, Gw, w, C;
    int nwy_o, nwx_o;     // windows of the merged grid
    int nwy_i, nwx_i;     // windows of the incoming grid
};

static MergeGeom make_geom(const rev_merge_cfg& c) {
    MergeGeom g;
    g.B = c.batch; g.Gh = c.grid_h; g.Gw = c.grid_w; g.w = c.window; g.C = c.d_in;
    g.nwy_i = c.grid_h / c.window; g.nwx_i = c.grid_w / c.window;
    g.nwy_o = c.grid_h / 2 / c.window; g.nwx_o = c.grid_w / 2 / c.window;
    return g;
}

// rows (window order, incoming grid) of the four neighbours that output row o (window order, merged grid) collects
__device__ __forceinline__ void merge_sources(const MergeGeom& g, int o, int src[4]) {
    const int ww = g.w * g.w;
    const int win = o / ww, in = o - win * ww;
    const int iy = in / g.w, ix = in - iy * g.w;
    const int per_img = g.nwy_o * g.nwx_o;
    const int b = win / per_img, wr = win - b * per_img;
    const int wy = wr / g.nwx_o, wx = wr - wy * g.nwx_o;
    const int y0 = 2 * (wy * g.w + iy), x0 = 2 * (wx * g.w + ix);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int y = y0 + (q >> 1), x = x0 + (q & 1);
        src[q] = ((b * g.nwy_i + y / g.w) * g.nwx_i + x / g.w) * ww + (y % g.w) * g.w + (x % g.w);
    }
}

// ---- gather + average + LayerNorm ---------------------------------------------------------------
// FUSED: the fused map z0 (activation type) is given; otherwise it is the average of X1 and X2, taken on the fly.
template <typename TA, typename TP, int MAXJ, bool FUSED>
__global__ __launch_bounds__(256) void merge_ln_fwd_kernel(const float* __restrict__ X1, const float* __restrict__ X2,
                                                           const TA* __restrict__ Z0,
                                                           const TP* __restrict__ gam, const TP* __restrict__ bet, float eps,
                                                           TA* __restrict__ n, float* __restrict__ stats, MergeGeom g, int Mo) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int o = blockIdx.x * 4 + wave;
    if (o >= Mo) return;
    const int C = g.C, D4 = 4 * C, nch = C;          // 4C floats = C chunks of 4
    int src[4];
    merge_sources(g, o, src);
    f4 v[MAXJ];
#pragma unroll
    for (int j = 0; j < MAXJ; ++j) {
        const int c = lane + 64 * j;
        if (c < nch) {
            const int q = (4 * c) / C, col = 4 * c - q * C;
            const int64_t off = (int64_t)src[q] * C + col;
            if (FUSED) {
                v[j] = load4(Z0 + off);
            } else {
                const f4 a = load4(X1 + off), b = load4(X2 + off);
                v[j] = {0.5f * (a.x + b.x), 0.5f * (a.y + b.y), 0.5f * (a.z + b.z), 0.5f * (a.w + b.w)};
            }
        }
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < MAXJ; ++j)
        if (lane + 64 * j < nch) s += (v[j].x + v[j].y) + (v[j].z + v[j].w);
    const float mean = wave_sum(s) / (float)D4;
    float qs = 0.f;
#pragma unroll
    for (int j = 0; j < MAXJ; ++j)
        if (lane + 64 * j < nch) {
            const float a0 = v[j].x - mean, a1 = v[j].y - mean, a2 = v[j].z - mean, a3 = v[j].w - mean;
            qs += (a0 * a0 + a1 * a1) + (a2 * a2 + a3 * a3);
        }
    const float rstd = 1.0f / sqrtf(wave_sum(qs) / (float)D4 + eps);
    TA* nr = n + (int64_t)o * D4;
#pragma unroll
    for (int j = 0; j < MAXJ; ++j) {
        const int c = lane + 64 * j;
        if (c < nch) {
            const f4 gg = load4(gam + 4 * c), bb = load4(bet + 4 * c);
            f4 r;
            r.x = (v[j].x - mean) * rstd * gg.x + bb.x;
            r.y = (v[j].y - mean) * rstd * gg.y + bb.y;
            r.z = (v[j].z - mean) * rstd * gg.z + bb.z;
            r.w = (v[j].w - mean) * rstd * gg.w + bb.w;
            store4(nr + 4 * c, r);
        }
    }
    if (lane == 0) {
        stats[2 * (int64_t)o] = mean;
        stats[2 * (int64_t)o + 1] = rstd;
    }
}

// ---- LayerNorm backward on the re-gathered row + scatter of the halves to both streams -------------
// Each block walks rows_per_block consecutive output rows (4 wavefronts, one row each at a time) and
// writes one partial row [d gamma | d beta], its wavefronts folded in wavefront order.
// FUSED: rows are re-gathered from the fused map z0 and their cotangent goes, whole, to dZ0 (activation type);
// otherwise from the average of X1 and X2, and half of it goes to each of dX1, dX2.
template <typename TA, typename TP, int MAXJ, bool FUSED>
__global__ __launch_bounds__(256) void merge_ln_bwd_kernel(const TA* __restrict__ dn, const float* __restrict__ X1,
                                                           const float* __restrict__ X2, const TA* __restrict__ Z0,
                                                           const float* __restrict__ stats,
                                                           const TP* __restrict__ gam, float* __restrict__ dX1,
                                                           float* __restrict__ dX2, TA* __restrict__ dZ0,
                                                           float* __restrict__ partial,
                                                           MergeGeom g, int Mo, int rows_per_block) {
    extern __shared__ float lds[];                   // [2 * 4C]
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int C = g.C, D4 = 4 * C, nch = C;
    f4 ag[MAXJ], ab[MAXJ], gg[MAXJ];
#pragma unroll
    for (int j = 0; j < MAXJ; ++j) {
        const int c = lane + 64 * j;
        gg[j] = (c < nch) ? load4(gam + 4 * c) : f4{0.f, 0.f, 0.f, 0.f};
        ag[j] = {0.f, 0.f, 0.f, 0.f};
        ab[j] = {0.f, 0.f, 0.f, 0.f};
    }
    const int row0 = blockIdx.x * rows_per_block;
    const int row1 = min(Mo, row0 + rows_per_block);
    for (int o = row0 + wave; o < row1; o += 4) {
        const float mean = stats[2 * (int64_t)o], rstd = stats[2 * (int64_t)o + 1];
        int src[4];
        merge_sources(g, o, src);
        f4 xh[MAXJ], dh[MAXJ];
        float c1 = 0.f, c2 = 0.f;
#pragma unroll
        for (int j = 0; j < MAXJ; ++j) {
            const int c = lane + 64 * j;
            if (c < nch) {
                const int q = (4 * c) / C, col = 4 * c - q * C;
                const int64_t off = (int64_t)src[q] * C + col;
                const f4 d = load4(dn + (int64_t)o * D4 + 4 * c);
                f4 zz;
                if (FUSED) {
                    zz = load4(Z0 + off);
                } else {
                    const f4 a = load4(X1 + off), b = load4(X2 + off);
                    zz = {0.5f * (a.x + b.x), 0.5f * (a.y + b.y), 0.5f * (a.z + b.z), 0.5f * (a.w + b.w)};
                }
                xh[j] = {(zz.x - mean) * rstd, (zz.y - mean) * rstd, (zz.z - mean) * rstd, (zz.w - mean) * rstd};
                ab[j].x += d.x; ab[j].y += d.y; ab[j].z += d.z; ab[j].w += d.w;
                ag[j].x += d.x * xh[j].x; ag[j].y += d.y * xh[j].y; ag[j].z += d.z * xh[j].z; ag[j].w += d.w * xh[j].w;
                dh[j] = {d.x * gg[j].x, d.y * gg[j].y, d.z * gg[j].z, d.w * gg[j].w};
                c1 += (dh[j].x + dh[j].y) + (dh[j].z + dh[j].w);
                c2 += (dh[j].x * xh[j].x + dh[j].y * xh[j].y) + (dh[j].z * xh[j].z + dh[j].w * xh[j].w);
            }
        }
        c1 = wave_sum(c1) / (float)D4;
        c2 = wave_sum(c2) / (float)D4;
        const float hr = FUSED ? rstd : 0.5f * rstd;
#pragma unroll
        for (int j = 0; j < MAXJ; ++j) {
            const int c = lane + 64 * j;
            if (c < nch) {
                const int q = (4 * c) / C, col = 4 * c - q * C;
                const int64_t off = (int64_t)src[q] * C + col;
                f4 r;
                r.x = hr * (dh[j].x - c1 - xh[j].x * c2);
                r.y = hr * (dh[j].y - c1 - xh[j].y * c2);
                r.z = hr * (dh[j].z - c1 - xh[j].z * c2);
                r.w = hr * (dh[j].w - c1 - xh[j].w * c2);
                if (FUSED) {
                    store4(dZ0 + off, r);
                } else {
                    store4(dX1 + off, r);
                    store4(dX2 + off, r);
                }
            }
        }
    }
    // fold the 4 wavefronts' column accumulators in wavefront order
    for (int w = 0; w < 4; ++w) {
        if (wave == w) {
#pragma unroll
            for (int j = 0; j < MAXJ; ++j) {
                const int c = lane + 64 * j;
                if (c < nch) {
                    float* pg = lds + 4 * c;
                    float* pb = lds + D4 + 4 * c;
                    if (w == 0) {
                        pg[0] = ag[j].x; pg[1] = ag[j].y; pg[2] = ag[j].z; pg[3] = ag[j].w;
                        pb[0] = ab[j].x; pb[1] = ab[j].y; pb[2] = ab[j].z; pb[3] = ab[j].w;
                    } else {
                        pg[0] += ag[j].x; pg[1] += ag[j].y; pg[2] += ag[j].z; pg[3] += ag[j].w;
                        pb[0] += ab[j].x; pb[1] += ab[j].y; pb[2] += ab[j].z; pb[3] += ab[j].w;
                    }
                }
            }
        }
        __syncthreads();
    }
    float* prow = partial + (int64_t)blockIdx.x * 2 * D4;
    for (int i = threadIdx.x; i < 2 * D4; i += 256) prow[i] = lds[i];
}

// dst = a + b, converted to the activation type
template <typename TA>
__global__ __launch_bounds__(256) void add2_kernel(const float* __restrict__ a, const float* __restrict__ b,
                                                   TA* __restrict__ dst, int64_t n4) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n4) {
        const f4 x = load4(a + 4 * i), y = load4(b + 4 * i);
        store4(dst + 4 * i, f4{x.x + y.x, x.y + y.y, x.z + y.z, x.w + y.w});
    }
}

// cat[m, 0:C] = X1[m, :], cat[m, C:2C] = X2[m, :], converted to the activation type
template <typename TA>
__global__ __launch_bounds__(256) void concat2_kernel(const float* __restrict__ X1, const float* __restrict__ X2,
                                                      TA* __restrict__ cat, int64_t M, int C4) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;       // one 4-element chunk of one source row
    if (i >= M * C4) return;
    const int64_t m = i / C4;
    const int c = (int)(i - m * C4);
    store4(cat + (m * 2 * C4 + c) * 4, load4(X1 + i * 4));
    store4(cat + (m * 2 * C4 + C4 + c) * 4, load4(X2 + i * 4));
}

// rows per block of the backward kernel: about 1024 blocks, at least 8 and at most 64 rows each
static int merge_rows_per_block(int Mo) {
    int rpb = ((Mo + 1023) / 1024 + 3) / 4 * 4;
    if (rpb < 8) rpb = 8;
    if (rpb > 64) rpb = 64;
    return rpb;
}

int64_t wgrad_partial_elems(int M, int N, int K);   // gemm_mfma.hip

// ---- workspace ---------------------------------------------------------------------------------
struct MergeLayout {
    int64_t n, stats, dob, dn, part_ln, part_wg, total;
    int64_t part_wg_elems;
    // fusion by a small MLP only: [X1 | X2], hidden pre-activation and activation, fused map, its cotangent, the
    // hidden cotangent (all [M, .] in the activation type), and the partial sums of the four parameter gradients
    int64_t cat, h, a, z0, dz0, dh, part_col[2], part_fw[2];
    int64_t part_fw_elems[2];
};
static MergeLayout merge_layout(const rev_merge_cfg& c) {
    MergeLayout L = {};
    const int64_t es = (c.mode == REV_MODE_BF16) ? 2 : 4;
    const int64_t Mo = (int64_t)c.batch * (c.grid_h / 2) * (c.grid_w / 2), C = c.d_in;
    int64_t pos = 0;
    auto take = [&](int64_t bytes) { int64_t at = pos; pos += (bytes + 255) / 256 * 256; return at; };
    L.n = take(Mo * 4 * C * es);
    L.stats = take(Mo * 2 * 4);
    L.dob = take(Mo * 2 * C * es);
    L.dn = take(Mo * 4 * C * es);
    const int rpb = merge_rows_per_block((int)Mo);
    L.part_ln = take(((Mo + rpb - 1) / rpb) * 8 * C * 4);
    L.part_wg_elems = (c.mode == REV_MODE_BF16) ? wgrad_partial_elems((int)Mo, (int)(2 * C), (int)(4 * C)) : 0;
    L.part_wg = take(L.part_wg_elems * 4);
    if (c.fusion == REV_FUSION_MLP) {
        const int64_t M = 4 * Mo;
        L.cat = take(M * 2 * C * es);
        L.h = take(M * C * es);
        L.a = take(M * C * es);
        L.z0 = take(M * C * es);
        L.dz0 = take(M * C * es);
        L.dh = take(M * C * es);
        L.part_col[0] = take(colsum_partial_elems((int)M, (int)C) * 4);
        L.part_col[1] = take(colsum_partial_elems((int)M, (int)C) * 4);
        L.part_fw_elems[0] = (c.mode == REV_MODE_BF16) ? wgrad_partial_elems((int)M, (int)C, (int)(2 * C)) : 0;
        L.part_fw_elems[1] = (c.mode == REV_MODE_BF16) ? wgrad_partial_elems((int)M, (int)C, (int)C) : 0;
        L.part_fw[0] = take((L.part_fw_elems[0] > 0 ? L.part_fw_elems[0] : 64) * 4);
        L.part_fw[1] = take((L.part_fw_elems[1] > 0 ? L.part_fw_elems[1] : 64) * 4);
    }
    L.total = pos;
    return L;
}

static int merge_check(const rev_merge_cfg* c) {
    if (!c) { set_error("merge cfg is null"); return REV_EINVAL; }
    if (c->batch <= 0 || c->grid_h <= 0 || c->grid_w <= 0 || c->window <= 0 || c->d_in <= 0) {
        set_error("merge cfg: every size must be positive"); return REV_EINVAL;
    }
    if (c->mode != REV_MODE_FP32 && c->mode != REV_MODE_BF16) { set_error("merge cfg: unknown mode"); return REV_EINVAL; }
    if (c->fusion != REV_FUSION_AVERAGE && c->fusion != REV_FUSION_MLP) { set_error("merge cfg: unknown fusion"); return REV_EINVAL; }
    if (c->grid_h % (2 * c->window) != 0 || c->grid_w % (2 * c->window) != 0) {
        set_error("merge cfg: grid_h and grid_w must be multiples of 2*window"); return REV_EINVAL;
    }
    if (c->d_in % 8 != 0) { set_error("merge cfg: d_in must be a multiple of 8"); return REV_EINVAL; }
    if (c->d_in > 2048) { set_error("merge cfg: d_in must be <= 2048"); return REV_EINVAL; }
    if ((int64_t)c->batch * c->grid_h * c->grid_w >= (1 << 24)) { set_error("merge cfg: batch*grid_h*grid_w must be < 2^24"); return REV_EINVAL; }
    if (!(c->ln_eps >= 0.f)) { set_error("merge cfg: ln_eps must be >= 0"); return REV_EINVAL; }
    return REV_OK;
}

#define RC(expr) do { int _rc = (expr); if (_rc != REV_OK) return _rc; } while (0)

template <typename T>
struct MergeRunner {
    static constexpr bool kBf16 = sizeof(T) == 2;
    rev_merge_cfg c;
    MergeLayout L;
    MergeGeom g;
    char* ws;
    const T* params;
    int Mo, C;

    MergeRunner(const rev_merge_cfg& cfg, const void* p, void* w)
        : c(cfg), L(merge_layout(cfg)), g(make_geom(cfg)), ws((char*)w), params((const T*)p) {
        Mo = c.batch * (c.grid_h / 2) * (c.grid_w / 2); C = c.d_in;
    }
    template <typename U> U* at(int64_t off) const { return reinterpret_cast<U*>(ws + off); }
    const T* gam() const { return params; }
    const T* bet() const { return params + 4 * C; }
    const T* W() const { return params + 8 * C; }
    // fusion MLP, behind the patch-merging parameters: Wa [C, 2C], ba [C], Wb [C, C], bb [C]
    int64_t off_wa() const { return (int64_t)8 * C + (int64_t)8 * C * C; }
    int64_t off_ba() const { return off_wa() + (int64_t)2 * C * C; }
    int64_t off_wb() const { return off_ba() + C; }
    int64_t off_bb() const { return off_wb() + (int64_t)C * C; }
    bool mlp() const { return c.fusion == REV_FUSION_MLP; }
    int Mi() const { return 4 * Mo; }

    // fusion by a small MLP: [X1 | X2] -> hidden (pre-activation h and a = gelu(h) are both kept) -> z0
    int fuse_mlp(hipStream_t s, const float* X1, const float* X2) {
        const int M = Mi();
        {
            const int64_t n4 = (int64_t)M * C / 4;
            ProfScope ps(K_CONVERT, s, (double)n4 * 4 * 2 * (4 + sizeof(T)));
            hipLaunchKernelGGL((concat2_kernel<T>), dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, s, X1, X2, at<T>(L.cat),
                               (int64_t)M, C / 4);
            REV_HIP(hipGetLastError());
        }
        Epi e = {}; e.kind = EPI_BIAS_GELU; e.out = at<T>(L.h); e.out2 = at<T>(L.a); e.bias = params + off_ba(); e.ldo = C; e.solo = true;
        Epi f = {}; f.kind = EPI_BIAS; f.out = at<T>(L.z0); f.bias = params + off_bb(); f.ldo = C; f.solo = true;
        if constexpr (kBf16) {
            RC(gemm_nt_bf16(s, at<T>(L.cat), 2 * C, params + off_wa(), 2 * C, M, C, 2 * C, e));
            return gemm_nt_bf16(s, at<T>(L.a), C, params + off_wb(), C, M, C, C, f);
        } else {
            RC(gemm_nt_f32(s, at<T>(L.cat), 2 * C, params + off_wa(), 2 * C, M, C, 2 * C, e));
            return gemm_nt_f32(s, at<T>(L.a), C, params + off_wb(), C, M, C, C, f);
        }
    }

    int gather_ln(hipStream_t s, const float* X1, const float* X2) {
        if (mlp()) RC(fuse_mlp(s, X1, X2));
        ProfScope ps(K_LN_FWD, s, (double)Mo * 4 * C * (8 + sizeof(T)));
        dim3 grid((Mo + 3) / 4), block(256);
        const T* z0 = mlp() ? at<T>(L.z0) : nullptr;
        switch (pick_maxj(4 * C)) {
#define CASE(J) case J:                                                                                                      \
            if (mlp()) hipLaunchKernelGGL((merge_ln_fwd_kernel<T, T, J, true>), grid, block, 0, s, X1, X2, z0, gam(), bet(),   \
                                          c.ln_eps, at<T>(L.n), at<float>(L.stats), g, Mo);                                    \
            else hipLaunchKernelGGL((merge_ln_fwd_kernel<T, T, J, false>), grid, block, 0, s, X1, X2, z0, gam(), bet(),        \
                                    c.ln_eps, at<T>(L.n), at<float>(L.stats), g, Mo);                                          \
            break;
            CASE(2) CASE(3) CASE(4) CASE(5) CASE(6) CASE(8) CASE(12) CASE(16) CASE(24) CASE(32)
#undef CASE
            default: set_error("merge: d_in too large"); return REV_EINVAL;
        }
        REV_HIP(hipGetLastError());
        return REV_OK;
    }

    int forward(hipStream_t s, const float* X1, const float* X2, float* out) {
        RC(gather_ln(s, X1, X2));
        Epi e = {}; e.kind = EPI_PLAIN_F32; e.outf = out; e.ldo = 2 * C; e.solo = true;
        if constexpr (kBf16) return gemm_nt_bf16(s, at<T>(L.n), 4 * C, W(), 4 * C, Mo, 2 * C, 4 * C, e);
        else return gemm_nt_f32(s, at<T>(L.n), 4 * C, W(), 4 * C, Mo, 2 * C, 4 * C, e);
    }

    int backward(hipStream_t s, const float* X1, const float* X2, const float* dA, const float* dB,
                 float* dX1, float* dX2, float* dparams) {
        RC(gather_ln(s, X1, X2));
        {
            const int64_t n4 = (int64_t)Mo * 2 * C / 4;
            ProfScope ps(K_CONVERT, s, (double)n4 * 4 * (8 + sizeof(T)));
            hipLaunchKernelGGL((add2_kernel<T>), dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, s, dA, dB, at<T>(L.dob), n4);
            REV_HIP(hipGetLastError());
        }
        RedSeg segs[2];
        float* dW = dparams + 8 * C;
        Epi e = {}; e.kind = EPI_PLAIN; e.out = at<T>(L.dn); e.ldo = 4 * C; e.solo = true;
        if constexpr (kBf16) {
            RC(gemm_wgrad_bf16(s, at<T>(L.dob), 2 * C, at<T>(L.n), 4 * C, Mo, 2 * C, 4 * C, dW, at<float>(L.part_wg), L.part_wg_elems, &segs[0]));
            RC(gemm_nn_bf16(s, at<T>(L.dob), 2 * C, W(), 4 * C, Mo, 4 * C, 2 * C, e));
        } else {
            RC(gemm_wgrad_f32(s, at<T>(L.dob), 2 * C, at<T>(L.n), 4 * C, Mo, 2 * C, 4 * C, dW, nullptr, 0, &segs[0]));
            RC(gemm_nn_f32(s, at<T>(L.dob), 2 * C, W(), 4 * C, Mo, 4 * C, 2 * C, e));
        }
        const int rpb = merge_rows_per_block(Mo);
        const int nblk = (Mo + rpb - 1) / rpb;
        {
            ProfScope ps(K_LN_BWD, s, (double)Mo * 4 * C * (sizeof(T) + 8 + 8));
            dim3 grid(nblk), block(256);
            const size_t shmem = (size_t)8 * C * sizeof(float);
            switch (pick_maxj(4 * C)) {
#define CASE(J) case J:                                                                                                      \
                if (mlp()) hipLaunchKernelGGL((merge_ln_bwd_kernel<T, T, J, true>), grid, block, shmem, s, at<T>(L.dn), X1, X2, \
                                              at<T>(L.z0), at<float>(L.stats), gam(), dX1, dX2, at<T>(L.dz0),                  \
                                              at<float>(L.part_ln), g, Mo, rpb);                                               \
                else hipLaunchKernelGGL((merge_ln_bwd_kernel<T, T, J, false>), grid, block, shmem, s, at<T>(L.dn), X1, X2,     \
                                        (const T*)nullptr, at<float>(L.stats), gam(), dX1, dX2, (T*)nullptr,                  \
                                        at<float>(L.part_ln), g, Mo, rpb);                                                     \
                break;
                CASE(2) CASE(3) CASE(4) CASE(5) CASE(6) CASE(8) CASE(12) CASE(16) CASE(24) CASE(32)
#undef CASE
                default: set_error("merge: d_in too large"); return REV_EINVAL;
            }
            REV_HIP(hipGetLastError());
        }
        // d gamma | d beta are adjacent in the packed layout
        segs[1] = {at<float>(L.part_ln), dparams, nullptr, (int64_t)8 * C, (int64_t)8 * C, (int64_t)8 * C, nblk};
        if (segs[0].P > 0) RC(reduce_multi(s, segs, 2));
        else RC(reduce_multi(s, &segs[1], 1));
        return mlp() ? fuse_mlp_backward(s, dX1, dX2, dparams) : REV_OK;
    }

    // dz0 (cotangent of the fused map) -> dX1, dX2 and the gradients of the fusion MLP; cat, h, a are those
    // the forward half of this call left in the workspace
    int fuse_mlp_backward(hipStream_t s, float* dX1, float* dX2, float* dparams) {
        const int M = Mi();
        T* dz0 = at<T>(L.dz0);
        T* dh = at<T>(L.dh);
        RedSeg segs[4];
        int nseg = 0;
        RedSeg wseg[2];
        // output layer: db = column sums, dWb = dz0^T * a, da = dz0 * Wb, dh = da * gelu'(h)
        RC(colsum<T>(s, dz0, C, M, C, dparams + off_bb(), at<float>(L.part_col[0]), &segs[nseg++]));
        Epi e = {}; e.kind = EPI_GELU_BWD; e.out = dh; e.aux = at<T>(L.h); e.ldo = C; e.solo = true;
        Epi x1 = {}; x1.kind = EPI_PLAIN_F32; x1.outf = dX1; x1.ldo = C; x1.solo = true;
        Epi x2 = x1; x2.outf = dX2;
        if constexpr (kBf16) {
            RC(gemm_wgrad_bf16(s, dz0, C, at<T>(L.a), C, M, C, C, dparams + off_wb(), at<float>(L.part_fw[1]), L.part_fw_elems[1], &wseg[1]));
            RC(gemm_nn_bf16(s, dz0, C, params + off_wb(), C, M, C, C, e));
        } else {
            RC(gemm_wgrad_f32(s, dz0, C, at<T>(L.a), C, M, C, C, dparams + off_wb(), nullptr, 0, &wseg[1]));
            RC(gemm_nn_f32(s, dz0, C, params + off_wb(), C, M, C, C, e));
        }
        // hidden layer: db = column sums of dh, dWa = dh^T * [X1 | X2], [dX1 | dX2] = dh * Wa (one GEMM per half:
        // the two streams' cotangents are separate buffers)
        RC(colsum<T>(s, dh, C, M, C, dparams + off_ba(), at<float>(L.part_col[1]), &segs[nseg++]));
        if constexpr (kBf16) {
            RC(gemm_wgrad_bf16(s, dh, C, at<T>(L.cat), 2 * C, M, C, 2 * C, dparams + off_wa(), at<float>(L.part_fw[0]), L.part_fw_elems[0], &wseg[0]));
            RC(gemm_nn_bf16(s, dh, C, params + off_wa(), 2 * C, M, C, C, x1));
            RC(gemm_nn_bf16(s, dh, C, params + off_wa() + C, 2 * C, M, C, C, x2));
        } else {
            RC(gemm_wgrad_f32(s, dh, C, at<T>(L.cat), 2 * C, M, C, 2 * C, dparams + off_wa(), nullptr, 0, &wseg[0]));
            RC(gemm_nn_f32(s, dh, C, params + off_wa(), 2 * C, M, C, C, x1));
            RC(gemm_nn_f32(s, dh, C, params + off_wa() + C, 2 * C, M, C, C, x2));
        }
        for (int w = 0; w < 2; ++w)
            if (wseg[w].P > 0) segs[nseg++] = wseg[w];
        return reduce_multi(s, segs, nseg);
    }
};

}  // namespace rev

using namespace rev;

extern "C" {

int rev_merge_check_cfg(const rev_merge_cfg* cfg) { return merge_check(cfg); }

int64_t rev_merge_param_count(const rev_merge_cfg* cfg) {
    if (merge_check(cfg) != REV_OK) return REV_EINVAL;
    const int64_t C = cfg->d_in;
    return 8 * C + 8 * C * C + (cfg->fusion == REV_FUSION_MLP ? 3 * C * C + 2 * C : 0);
}

int64_t rev_merge_workspace_bytes(const rev_merge_cfg* cfg) {
    if (merge_check(cfg) != REV_OK) return REV_EINVAL;
    return merge_layout(*cfg).total;
}

static int merge_common(const rev_merge_cfg* cfg, const void* ws, int64_t ws_bytes) {
    RC(merge_check(cfg));
    if (!ws) { set_error("workspace is null"); return REV_EINVAL; }
    if (((uintptr_t)ws & 255) != 0) { set_error("workspace must be 256-byte aligned"); return REV_EINVAL; }
    const MergeLayout L = merge_layout(*cfg);
    if (ws_bytes < L.total) {
        set_error("workspace too small: need " + std::to_string(L.total) + " bytes, got " + std::to_string(ws_bytes));
        return REV_EWORKSPACE;
    }
    return REV_OK;
}

int rev_merge_forward(const rev_merge_cfg* cfg, const void* params, const float* X1, const float* X2, float* out,
                      void* workspace, int64_t workspace_bytes, void* stream) {
    RC(merge_common(cfg, workspace, workspace_bytes));
    if (!params || !X1 || !X2 || !out) { set_error("a required pointer is null"); return REV_EINVAL; }
    if ((((uintptr_t)params | (uintptr_t)X1 | (uintptr_t)X2 | (uintptr_t)out) & 15) != 0) {
        set_error("every buffer must be 16-byte aligned"); return REV_EINVAL;
    }
    hipStream_t s = (hipStream_t)stream;
    if (cfg->mode == REV_MODE_BF16) { MergeRunner<bf16> r(*cfg, params, workspace); return r.forward(s, X1, X2, out); }
    MergeRunner<float> r(*cfg, params, workspace);
    return r.forward(s, X1, X2, out);
}

int rev_merge_backward(const rev_merge_cfg* cfg, const void* params, const float* X1, const float* X2,
                       const float* dOutA, const float* dOutB, float* dX1, float* dX2, float* dparams,
                       void* workspace, int64_t workspace_bytes, void* stream) {
    RC(merge_common(cfg, workspace, workspace_bytes));
    if (!params || !X1 || !X2 || !dOutA || !dOutB || !dX1 || !dX2 || !dparams) {
        set_error("a required pointer is null"); return REV_EINVAL;
    }
    if ((((uintptr_t)params | (uintptr_t)X1 | (uintptr_t)X2 | (uintptr_t)dOutA | (uintptr_t)dOutB | (uintptr_t)dX1 |
          (uintptr_t)dX2 | (uintptr_t)dparams) & 15) != 0) {
        set_error("every buffer must be 16-byte aligned"); return REV_EINVAL;
    }
    hipStream_t s = (hipStream_t)stream;
    if (cfg->mode == REV_MODE_BF16) {
        MergeRunner<bf16> r(*cfg, params, workspace);
        return r.backward(s, X1, X2, dOutA, dOutB, dX1, dX2, dparams);
    }
    MergeRunner<float> r(*cfg, params, workspace);
    return r.backward(s, X1, X2, dOutA, dOutB, dX1, dX2, dparams);
}

}  // extern "C"
