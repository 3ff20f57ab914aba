// Memory-bound kernels: LayerNorm forward / backward, column sums, fixed-order
// reductions, dtype conversion.  One wavefront (64 lanes) owns one
// row at a time and keeps it in registers; row statistics are wavefront
// reductions; column statistics (d gamma, d beta, bias gradients) are summed in
// a fixed order so that results do not depend on scheduling.
#include "common.h"
#include "rowwise.h"

namespace rev {

// ---- LayerNorm forward -----------------------------------------------------------
// Lane l of the row's wavefront holds 4-element chunks l, l+64, ... (MAXJ of them).  A wavefront
// handles two rows (rows w and w + M/2-ish apart are both requested before either is reduced), so
// every lane has two independent memory round trips in flight.
template <typename TA, typename TP, int MAXJ>
__global__ __launch_bounds__(256) void ln_fwd_kernel(const float* __restrict__ x, const TP* __restrict__ g,
                                                     const TP* __restrict__ b, float eps,
                                                     TA* __restrict__ y, float* __restrict__ stats,
                                                     int M, int D) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int half = (M + 1) >> 1;
    const int r0 = blockIdx.x * 4 + wave;          // rows r0 and r0 + half
    if (r0 >= half) return;
    const int nch = D >> 2;
    int rows[2] = {r0, r0 + half};
    const bool live1 = rows[1] < M;
    f4 v[2][MAXJ];
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const float* xr = x + (int64_t)rows[k] * D;
        if (k == 1 && !live1) break;
#pragma unroll
        for (int j = 0; j < MAXJ; ++j) {
            int c = lane + 64 * j;
            if (c < nch) v[k][j] = load4(xr + 4 * c);
        }
    }
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        if (k == 1 && !live1) break;
        float s = 0.f;
#pragma unroll
        for (int j = 0; j < MAXJ; ++j) {
            int c = lane + 64 * j;
            if (c < nch) s += (v[k][j].x + v[k][j].y) + (v[k][j].z + v[k][j].w);
        }
        const float mean = wave_sum(s) / (float)D;
        float q = 0.f;
#pragma unroll
        for (int j = 0; j < MAXJ; ++j) {
            int c = lane + 64 * j;
            if (c < nch) {
                float a0 = v[k][j].x - mean, a1 = v[k][j].y - mean, a2 = v[k][j].z - mean, a3 = v[k][j].w - mean;
                q += (a0 * a0 + a1 * a1) + (a2 * a2 + a3 * a3);
            }
        }
        const float rstd = 1.0f / sqrtf(wave_sum(q) / (float)D + eps);
        TA* yr = y + (int64_t)rows[k] * D;
#pragma unroll
        for (int j = 0; j < MAXJ; ++j) {
            int c = lane + 64 * j;
            if (c < nch) {
                f4 gg = load4(g + 4 * c), bb = load4(b + 4 * c), o;
                o.x = (v[k][j].x - mean) * rstd * gg.x + bb.x;
                o.y = (v[k][j].y - mean) * rstd * gg.y + bb.y;
                o.z = (v[k][j].z - mean) * rstd * gg.z + bb.z;
                o.w = (v[k][j].w - mean) * rstd * gg.w + bb.w;
                store4(yr + 4 * c, o);
            }
        }
        if (lane == 0) {
            stats[2 * (int64_t)rows[k]] = mean;
            stats[2 * (int64_t)rows[k] + 1] = rstd;
        }
    }
}

template <typename TA, typename TP>
int ln_forward(hipStream_t s, const float* x, const TP* g, const TP* b, float eps,
               TA* y, float* stats, int M, int D) {
    ProfScope ps(K_LN_FWD, s, (double)M * D * (4 + sizeof(TA)));
    dim3 grid(((M + 1) / 2 + 3) / 4), block(256);
    switch (pick_maxj(D)) {
#define CASE(J) case J: hipLaunchKernelGGL((ln_fwd_kernel<TA, TP, J>), grid, block, 0, s, x, g, b, eps, y, stats, M, D); break;
        CASE(2) CASE(3) CASE(4) CASE(5) CASE(6) CASE(8) CASE(12) CASE(16) CASE(24) CASE(32)
#undef CASE
        default: set_error("ln_forward: d_model too large"); return REV_EINVAL;
    }
    REV_HIP(hipGetLastError());
    return REV_OK;
}
template int ln_forward<float, float>(hipStream_t, const float*, const float*, const float*, float, float*, float*, int, int);
template int ln_forward<bf16, bf16>(hipStream_t, const float*, const bf16*, const bf16*, float, bf16*, float*, int, int);

// ---- LayerNorm backward + residual-gradient add -----------------------------------------
// out = r + rstd * (dxh - mean(dxh) - xhat * mean(dxh * xhat)),  dxh = dn * g.
// Each block walks LNB_ROWS consecutive rows (4 wavefronts, one row each at a
// time); per-lane column accumulators for d gamma, d beta and the column sums of
// `out` itself (the bias gradient of the linear map that `out` is the cotangent
// of) are folded across the 4 wavefronts in LDS in wavefront order and written
// as one partial row [dgamma | dbeta | colsum(out)] per block.
constexpr int LNB_ROWS = 32;
// Rows per block (a multiple of 4): LNB_ROWS for 32 k rows and more; fewer, down to 8, for shorter
// inputs so that about 1024 blocks (4 per CU) are in flight; more once LNB_ROWS would give above 2048
// partial rows.
static int ln_bwd_rows_per_block(int M) {
    int rpb = LNB_ROWS;
    if ((M + rpb - 1) / rpb > 2048) rpb = (((M + 2047) / 2048) + 3) / 4 * 4;
    else if (M < 1024 * LNB_ROWS) rpb = ((M + 1023) / 1024 + 3) / 4 * 4;
    if (rpb < 8) rpb = 8;
    return rpb;
}

// Rows of 1024 floats and more (4+ register chunks per lane): the three column accumulators of a
// wavefront live in its own slice of LDS instead of registers (lane-private slots, no synchronisation),
// which roughly halves the register count and doubles the wavefronts in flight.
template <int MAXJ> struct LnBwdCfg { static constexpr bool ACC_LDS = (MAXJ >= 4 && MAXJ <= 8); };

template <typename TA, typename TP, int MAXJ>
__global__ __launch_bounds__(256) void ln_bwd_kernel(const TA* __restrict__ dn, const float* __restrict__ x,
                                                     const float* __restrict__ stats, const TP* __restrict__ g,
                                                     const float* __restrict__ r, float* __restrict__ out,
                                                     TA* __restrict__ outb, float* __restrict__ partial,
                                                     int M, int D, int rows_per_block) {
    constexpr bool ACC_LDS = LnBwdCfg<MAXJ>::ACC_LDS;
    extern __shared__ float lds[];   // [3 * D], or [4][3 * D] with ACC_LDS
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int nch = D >> 2;
    constexpr int NACC = ACC_LDS ? 1 : MAXJ;
    f4 ag[NACC], ab[NACC], ao[NACC], gg[MAXJ];
    float* wacc = lds + (ACC_LDS ? wave * 3 * D : 0);            // [dgamma | dbeta | colsum(out)] of this wavefront
#pragma unroll
    for (int j = 0; j < MAXJ; ++j) {
        int c = lane + 64 * j;
        gg[j] = (c < nch) ? load4(g + 4 * c) : f4{0.f, 0.f, 0.f, 0.f};
        if (ACC_LDS) {
            if (c < nch) {
                const f4 z = {0.f, 0.f, 0.f, 0.f};
                *reinterpret_cast<f4*>(wacc + 4 * c) = z;
                *reinterpret_cast<f4*>(wacc + D + 4 * c) = z;
                *reinterpret_cast<f4*>(wacc + 2 * D + 4 * c) = z;
            }
        } else {
            ag[j % NACC] = {0.f, 0.f, 0.f, 0.f};
            ab[j % NACC] = {0.f, 0.f, 0.f, 0.f};
            ao[j % NACC] = {0.f, 0.f, 0.f, 0.f};
        }
    }
    const int row0 = blockIdx.x * rows_per_block;
    const int row1 = min(M, row0 + rows_per_block);
    for (int row = row0 + wave; row < row1; row += 4) {
        const float mean = stats[2 * (int64_t)row], rstd = stats[2 * (int64_t)row + 1];
        const int64_t base = (int64_t)row * D;
        f4 xh[MAXJ], dh[MAXJ], rv[MAXJ];
        float c1 = 0.f, c2 = 0.f;
        // all three input rows are requested up front: one memory round trip per row, not two
#pragma unroll
        for (int j = 0; j < MAXJ; ++j) {
            int c = lane + 64 * j;
            if (c < nch) rv[j] = load4(r + base + 4 * c);
        }
#pragma unroll
        for (int j = 0; j < MAXJ; ++j) {
            int c = lane + 64 * j;
            if (c < nch) {
                f4 xv = load4(x + base + 4 * c), d = load4(dn + base + 4 * c);
                xh[j] = {(xv.x - mean) * rstd, (xv.y - mean) * rstd, (xv.z - mean) * rstd, (xv.w - mean) * rstd};
                if (ACC_LDS) {
                    f4 b0 = *reinterpret_cast<f4*>(wacc + D + 4 * c), g0 = *reinterpret_cast<f4*>(wacc + 4 * c);
                    b0.x += d.x; b0.y += d.y; b0.z += d.z; b0.w += d.w;
                    g0.x += d.x * xh[j].x; g0.y += d.y * xh[j].y; g0.z += d.z * xh[j].z; g0.w += d.w * xh[j].w;
                    *reinterpret_cast<f4*>(wacc + D + 4 * c) = b0;
                    *reinterpret_cast<f4*>(wacc + 4 * c) = g0;
                } else {
                    ab[j % NACC].x += d.x; ab[j % NACC].y += d.y; ab[j % NACC].z += d.z; ab[j % NACC].w += d.w;
                    ag[j % NACC].x += d.x * xh[j].x; ag[j % NACC].y += d.y * xh[j].y;
                    ag[j % NACC].z += d.z * xh[j].z; ag[j % NACC].w += d.w * xh[j].w;
                }
                dh[j] = {d.x * gg[j].x, d.y * gg[j].y, d.z * gg[j].z, d.w * gg[j].w};
                c1 += (dh[j].x + dh[j].y) + (dh[j].z + dh[j].w);
                c2 += (dh[j].x * xh[j].x + dh[j].y * xh[j].y) + (dh[j].z * xh[j].z + dh[j].w * xh[j].w);
            }
        }
        c1 = wave_sum(c1) / (float)D;
        c2 = wave_sum(c2) / (float)D;
#pragma unroll
        for (int j = 0; j < MAXJ; ++j) {
            int c = lane + 64 * j;
            if (c < nch) {
                f4 o;
                o.x = rv[j].x + rstd * (dh[j].x - c1 - xh[j].x * c2);
                o.y = rv[j].y + rstd * (dh[j].y - c1 - xh[j].y * c2);
                o.z = rv[j].z + rstd * (dh[j].z - c1 - xh[j].z * c2);
                o.w = rv[j].w + rstd * (dh[j].w - c1 - xh[j].w * c2);
                if (ACC_LDS) {
                    f4 o0 = *reinterpret_cast<f4*>(wacc + 2 * D + 4 * c);
                    o0.x += o.x; o0.y += o.y; o0.z += o.z; o0.w += o.w;
                    *reinterpret_cast<f4*>(wacc + 2 * D + 4 * c) = o0;
                } else {
                    ao[j % NACC].x += o.x; ao[j % NACC].y += o.y; ao[j % NACC].z += o.z; ao[j % NACC].w += o.w;
                }
                store4(out + base + 4 * c, o);
                if (outb) store4(outb + base + 4 * c, o);
            }
        }
    }
    float* prow = partial + (int64_t)blockIdx.x * 3 * D;
    if (ACC_LDS) {
        // fold the 4 wavefronts' slices in wavefront order
        __syncthreads();
        for (int i = threadIdx.x; i < 3 * D; i += 256)
            prow[i] = ((lds[i] + lds[3 * D + i]) + lds[6 * D + i]) + lds[9 * D + i];
        return;
    }
    // fold the 4 wavefronts' column accumulators in wavefront order
    for (int w = 0; w < 4; ++w) {
        if (wave == w) {
#pragma unroll
            for (int j = 0; j < MAXJ; ++j) {
                int c = lane + 64 * j;
                if (c < nch) {
                    float* pg = lds + 4 * c;
                    float* pb = lds + D + 4 * c;
                    float* po = lds + 2 * D + 4 * c;
                    if (w == 0) {
                        pg[0] = ag[j % NACC].x; pg[1] = ag[j % NACC].y; pg[2] = ag[j % NACC].z; pg[3] = ag[j % NACC].w;
                        pb[0] = ab[j % NACC].x; pb[1] = ab[j % NACC].y; pb[2] = ab[j % NACC].z; pb[3] = ab[j % NACC].w;
                        po[0] = ao[j % NACC].x; po[1] = ao[j % NACC].y; po[2] = ao[j % NACC].z; po[3] = ao[j % NACC].w;
                    } else {
                        pg[0] += ag[j % NACC].x; pg[1] += ag[j % NACC].y; pg[2] += ag[j % NACC].z; pg[3] += ag[j % NACC].w;
                        pb[0] += ab[j % NACC].x; pb[1] += ab[j % NACC].y; pb[2] += ab[j % NACC].z; pb[3] += ab[j % NACC].w;
                        po[0] += ao[j % NACC].x; po[1] += ao[j % NACC].y; po[2] += ao[j % NACC].z; po[3] += ao[j % NACC].w;
                    }
                }
            }
        }
        __syncthreads();
    }
    for (int i = threadIdx.x; i < 3 * D; i += 256) prow[i] = lds[i];
}

// out[i] = sum over p (ascending) of partial[p * stride + i]; 4 elements per thread.
// Elements at or beyond `split4` (in units of 4) go to out2 instead (nullable: dropped).
__device__ __forceinline__ void reduce_store(float* out, float* out2, int64_t split4, int64_t i, float4 acc) {
    if (i < split4) *reinterpret_cast<float4*>(out + 4 * i) = acc;
    else if (out2) *reinterpret_cast<float4*>(out2 + 4 * (i - split4)) = acc;
}

// ---- several fixed-order reductions in one launch ----------------------------------------------------
struct RedSegDev { const float* partial; float* out; float* out2; int64_t stride, n4, split4; int P, first_block; };
struct RedArgs { RedSegDev seg[RED_MAX_SEGS]; int nseg; };

// Segments with many partial rows (P > 32) use 16 row-lanes per group of 16 column quads, folded in
// lane order through LDS; the others one thread per column quad.  Either way the order is fixed.
__global__ __launch_bounds__(256) void reduce_multi_kernel(RedArgs a) {
    __shared__ float4 sh[256];
    int si = 0;
#pragma unroll
    for (int k = 1; k < RED_MAX_SEGS; ++k)
        if (k < a.nseg && (int)blockIdx.x >= a.seg[k].first_block) si = k;
    const RedSegDev g = a.seg[si];
    const int lb = blockIdx.x - g.first_block;
    if (g.P > 32) {
        const int cg = threadIdx.x & 15, pl = threadIdx.x >> 4;
        const int64_t i = (int64_t)lb * 16 + cg;
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        if (i < g.n4) {
            // 4 loads in flight per thread; the additions stay in ascending row order
            int p = pl;
            for (; p + 48 < g.P; p += 64) {
                const float* q = g.partial + (int64_t)p * g.stride + 4 * i;
                const float4 v0 = *reinterpret_cast<const float4*>(q);
                const float4 v1 = *reinterpret_cast<const float4*>(q + 16 * g.stride);
                const float4 v2 = *reinterpret_cast<const float4*>(q + 32 * g.stride);
                const float4 v3 = *reinterpret_cast<const float4*>(q + 48 * g.stride);
                acc.x += v0.x; acc.y += v0.y; acc.z += v0.z; acc.w += v0.w;
                acc.x += v1.x; acc.y += v1.y; acc.z += v1.z; acc.w += v1.w;
                acc.x += v2.x; acc.y += v2.y; acc.z += v2.z; acc.w += v2.w;
                acc.x += v3.x; acc.y += v3.y; acc.z += v3.z; acc.w += v3.w;
            }
            for (; p < g.P; p += 16) {
                float4 v = *reinterpret_cast<const float4*>(g.partial + (int64_t)p * g.stride + 4 * i);
                acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
            }
        }
        sh[threadIdx.x] = acc;
        __syncthreads();
        if (pl == 0 && i < g.n4) {
            for (int q = 1; q < 16; ++q) {
                float4 v = sh[q * 16 + cg];
                acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
            }
            reduce_store(g.out, g.out2, g.split4, i, acc);
        }
    } else {
        const int64_t i = (int64_t)lb * 256 + threadIdx.x;
        if (i >= g.n4) return;
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int p = 0; p < g.P; ++p) {
            float4 v = *reinterpret_cast<const float4*>(g.partial + (int64_t)p * g.stride + 4 * i);
            acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
        }
        reduce_store(g.out, g.out2, g.split4, i, acc);
    }
}

int reduce_multi(hipStream_t s, const RedSeg* segs, int nseg) {
    if (nseg <= 0) return REV_OK;
    if (nseg > RED_MAX_SEGS) { set_error("reduce_multi: too many segments"); return REV_EINVAL; }
    RedArgs a;
    a.nseg = nseg;
    int blocks = 0;
    double bytes = 0;
    for (int k = 0; k < nseg; ++k) {
        const RedSeg& g = segs[k];
        if (g.n % 4 != 0 || g.split % 4 != 0) { set_error("reduce_multi: lengths must be multiples of 4"); return REV_EINVAL; }
        const int64_t n4 = g.n / 4;
        a.seg[k] = {g.partial, g.out, g.out2, g.stride, n4, g.split / 4, g.P, blocks};
        blocks += (int)(g.P > 32 ? (n4 + 15) / 16 : (n4 + 255) / 256);
        bytes += (double)(g.P + 1) * g.n * 4;
    }
    ProfScope ps(K_REDUCE, s, bytes);
    hipLaunchKernelGGL(reduce_multi_kernel, dim3(blocks), dim3(256), 0, s, a);
    REV_HIP(hipGetLastError());
    return REV_OK;
}

int64_t ln_bwd_partial_elems(int M, int D) {
    const int rpb = ln_bwd_rows_per_block(M);
    return (int64_t)((M + rpb - 1) / rpb) * 3 * D;
}

template <typename TA, typename TP>
int ln_backward(hipStream_t s, const TA* dn, const float* x, const float* stats, const TP* g,
                const float* r, float* out, TA* outb, float* dgb, float* dbias,
                float* partial, int M, int D, RedSeg* defer) {
    const int rpb = ln_bwd_rows_per_block(M);
    const int nblk = (M + rpb - 1) / rpb;
    {
        ProfScope ps(K_LN_BWD, s, (double)M * D * (sizeof(TA) + 4 + 4 + 4 + (outb ? sizeof(TA) : 0)));
        dim3 grid(nblk), block(256);
        switch (pick_maxj(D)) {
#define CASE(J) case J: {                                                                                            \
            auto kern = ln_bwd_kernel<TA, TP, J>;                                                                       \
            constexpr int copies = LnBwdCfg<J>::ACC_LDS ? 4 : 1;                                                        \
            const size_t shmem = (size_t)copies * 3 * D * sizeof(float);                                                \
            static LdsLimit lim;                                                                                        \
            if (int rc = lim.ensure(reinterpret_cast<const void*>(kern), copies * 3 * 64 * J * 16)) return rc;          \
            hipLaunchKernelGGL(kern, grid, block, shmem, s, dn, x, stats, g, r, out, outb, partial, M, D, rpb);     \
        } break;
            CASE(2) CASE(3) CASE(4) CASE(5) CASE(6) CASE(8) CASE(12) CASE(16) CASE(24) CASE(32)
#undef CASE
            default: set_error("ln_backward: d_model too large"); return REV_EINVAL;
        }
        REV_HIP(hipGetLastError());
    }
    // partial rows are [dgamma(D) | dbeta(D) | colsum(out)(D)]; gamma and beta gradients are adjacent in dgb
    const RedSeg seg = {partial, dgb, dbias, 3 * (int64_t)D, 3 * (int64_t)D, 2 * (int64_t)D, nblk};
    if (defer) { *defer = seg; return REV_OK; }
    return reduce_multi(s, &seg, 1);
}
template int ln_backward<float, float>(hipStream_t, const float*, const float*, const float*, const float*, const float*, float*, float*, float*, float*, float*, int, int, RedSeg*);
template int ln_backward<bf16, bf16>(hipStream_t, const bf16*, const float*, const float*, const bf16*, const float*, float*, bf16*, float*, float*, float*, int, int, RedSeg*);

// ---- column sums (bias gradients) --------------------------------------------------------
// grid (column tiles of 256, row chunks); each wavefront sums a quarter of the
// block's rows for its 256 columns, the 4 wavefronts are folded in order.
template <typename T>
__global__ __launch_bounds__(256) void colsum_kernel(const T* __restrict__ in, int64_t ld, int M, int N,
                                                     int rows_per_block, float* __restrict__ partial) {
    __shared__ float lds[4][256];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int col = blockIdx.x * 256 + lane * 4;
    const int row0 = blockIdx.y * rows_per_block;
    const int row1 = min(M, row0 + rows_per_block);
    f4 acc = {0.f, 0.f, 0.f, 0.f};
    if (col < N) {
        for (int row = row0 + wave; row < row1; row += 4) {
            f4 v = load4(in + (int64_t)row * ld + col);
            acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
        }
    }
    lds[wave][lane * 4 + 0] = acc.x; lds[wave][lane * 4 + 1] = acc.y;
    lds[wave][lane * 4 + 2] = acc.z; lds[wave][lane * 4 + 3] = acc.w;
    __syncthreads();
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c < N) {
        float v = ((lds[0][threadIdx.x] + lds[1][threadIdx.x]) + lds[2][threadIdx.x]) + lds[3][threadIdx.x];
        partial[(int64_t)blockIdx.y * N + c] = v;
    }
}

static int colsum_chunks(int M, int N) {
    int tiles = (N + 255) / 256;
    int P = (2048 + tiles - 1) / tiles;
    int maxP = (M + 15) / 16;
    if (P > maxP) P = maxP;
    if (P < 1) P = 1;
    return P;
}
int64_t colsum_partial_elems(int M, int N) { return (int64_t)colsum_chunks(M, N) * N; }

template <typename T>
int colsum(hipStream_t s, const T* in, int64_t ld, int M, int N, float* out, float* partial, RedSeg* defer) {
    int P = colsum_chunks(M, N);
    int rpb = (M + P - 1) / P;
    P = (M + rpb - 1) / rpb;
    {
        ProfScope ps(K_COLSUM, s, (double)M * N * sizeof(T));
        dim3 grid((N + 255) / 256, P), block(256);
        hipLaunchKernelGGL((colsum_kernel<T>), grid, block, 0, s, in, ld, M, N, rpb, partial);
        REV_HIP(hipGetLastError());
    }
    const RedSeg g = {partial, out, nullptr, (int64_t)N, (int64_t)N, (int64_t)N, P};
    if (defer) { *defer = g; return REV_OK; }
    return reduce_multi(s, &g, 1);
}
template int colsum<float>(hipStream_t, const float*, int64_t, int, int, float*, float*, RedSeg*);
template int colsum<bf16>(hipStream_t, const bf16*, int64_t, int, int, float*, float*, RedSeg*);

// ---- conversion ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void cvt_kernel(const float* __restrict__ in, bf16* __restrict__ out, int64_t n4) {
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n4) store4(out + 4 * i, load4(in + 4 * i));
}
int convert_f32_to_bf16(hipStream_t s, const float* in, bf16* out, int64_t n) {
    if (n % 4 != 0) { set_error("convert: length must be a multiple of 4"); return REV_EINVAL; }
    ProfScope ps(K_CONVERT, s, (double)n * 6);
    int64_t n4 = n / 4;
    hipLaunchKernelGGL(cvt_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, s, in, out, n4);
    REV_HIP(hipGetLastError());
    return REV_OK;
}

}  // namespace rev
