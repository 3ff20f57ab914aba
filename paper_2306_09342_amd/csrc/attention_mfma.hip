// bf16 softmax attention on the matrix cores: forward (flash-style, log-sum-exp
// saved) and backward in two passes, each free of atomics so that every sum has
// a fixed order:
//   pass 1  one wavefront owns 32 query rows, streams key/value tiles:  dQ, delta
//   pass 2  one wavefront owns 32 key rows, streams query/dO tiles:     dK, dV
//
// The score tile is always produced with the OWNED index on the accumulator's
// column (lane) axis: S^T[key, q] in the forward and in pass 1, S[q, key] in
// pass 2.  Row statistics of the owned index are then per-lane scalars, and the
// probability tile, converted to bf16 where it sits, is directly the B operand
// of the next product; the streamed operand of that product is read from its
// row-major LDS tile with the LDS transpose read.  No tile is ever transposed
// through memory or shuffled across lanes.
//
// Heads of 64 or 32 features and up to 256 tokens run both backward passes in ONE workgroup per head
// (attn_bwd_fused): Q, K, V and dO of the head go to LDS once, with direct-to-LDS loads, and the row statistics travel from pass 1 to pass 2
// through LDS.  Other shapes use the two kernels.
#include "mfma.h"

namespace rev {

constexpr int AT_ROWS = 64;     // streamed rows per LDS tile

template <int DHP> struct AtCfg {
    static constexpr int KS = DHP / 16;          // contraction steps over the head dim
    static constexpr int DT = DHP / 32;          // 32-wide output tiles over the head dim
    static constexpr int PITCH = DHP + 8;        // LDS row pitch (elements)
    static constexpr int CH = DHP / 8;           // 16-byte chunks per row
};

// B-operand fragments of 32 owned rows straight from global memory:
// lane (r = l%32, g) takes X[row0 + r][16*ks + 8g .. +7]; rows are clamped, columns >= dh read as zero.
template <int DHP>
__device__ __forceinline__ void load_owned(const bf16* __restrict__ base, int64_t ld, int row0, int nrows, int dh,
                                           int lane, bf16x8_t (&frag)[DHP / 16]) {
    const int r = min(row0 + (lane & 31), nrows - 1);
    const bf16* p = base + (int64_t)r * ld + 8 * (lane >> 5);
#pragma unroll
    for (int ks = 0; ks < DHP / 16; ++ks) {
        const int c = 16 * ks + 8 * (lane >> 5);
        u32x4_t v = {0u, 0u, 0u, 0u};
        if (c < dh) v = *reinterpret_cast<const u32x4_t*>(p + 16 * ks);
        union { u32x4_t u; bf16x8_t b; } cv;
        cv.u = v;
        frag[ks] = cv.b;
    }
}

// Cooperative load of `trows` rows [row0, row0+trows) of a [nrows, ld] matrix into an LDS tile;
// rows >= nrows and columns >= dh are zero-filled.
template <int DHP>
__device__ __forceinline__ void load_tile(uint16_t* tile, const bf16* __restrict__ base, int64_t ld, int row0,
                                          int nrows, int dh, int trows) {
    constexpr int CH = AtCfg<DHP>::CH, PITCH = AtCfg<DHP>::PITCH;
    for (int idx = threadIdx.x; idx < trows * CH; idx += blockDim.x) {
        const int row = idx / CH, ch = idx % CH;
        const int gr = row0 + row;
        u32x4_t v = {0u, 0u, 0u, 0u};
        if (gr < nrows && ch * 8 < dh) v = *reinterpret_cast<const u32x4_t*>(base + (int64_t)gr * ld + ch * 8);
        *reinterpret_cast<u32x4_t*>(tile + row * PITCH + ch * 8) = v;
    }
}

// The same load in two halves, for the streamed mode (64-row tiles): the global loads of the NEXT
// tile are issued into registers before the products of the current one and stored to LDS after them,
// so their latency is covered by the matrix-core work instead of being waited for at every tile.
// A thread holds DHP / 32 16-byte pieces of one tile (enough for 64 rows with 4 or more wavefronts);
// the launcher picks the plain-load instantiation for smaller workgroups.
template <int DHP> struct TilePre {
    static constexpr int N = DHP / 32;
    u32x4_t v[N];
};

template <int DHP>
__device__ __forceinline__ void tile_fetch(TilePre<DHP>& t, const bf16* __restrict__ base, int64_t ld, int row0,
                                           int nrows, int dh) {
    constexpr int CH = AtCfg<DHP>::CH;
#pragma unroll
    for (int i = 0; i < TilePre<DHP>::N; ++i) {
        const int idx = threadIdx.x + i * blockDim.x;
        const int row = idx / CH, ch = idx % CH;
        const int gr = row0 + row;
        u32x4_t v = {0u, 0u, 0u, 0u};
        if (idx < AT_ROWS * CH && gr < nrows && ch * 8 < dh) v = *reinterpret_cast<const u32x4_t*>(base + (int64_t)gr * ld + ch * 8);
        t.v[i] = v;
    }
}
template <int DHP>
__device__ __forceinline__ void tile_store(uint16_t* tile, const TilePre<DHP>& t) {
    constexpr int CH = AtCfg<DHP>::CH, PITCH = AtCfg<DHP>::PITCH;
#pragma unroll
    for (int i = 0; i < TilePre<DHP>::N; ++i) {
        const int idx = threadIdx.x + i * blockDim.x;
        const int row = idx / CH, ch = idx % CH;
        if (idx < AT_ROWS * CH) *reinterpret_cast<u32x4_t*>(tile + row * PITCH + ch * 8) = t.v[i];
    }
}

__device__ __forceinline__ bf16x8_t pack8(const float* p) {
    bf16x8_t r;
#pragma unroll
    for (int e = 0; e < 8; ++e) r[e] = (__bf16)p[e];
    return r;
}

__device__ __forceinline__ void store4_bf16(bf16* p, float a, float b, float c, float d) {
    typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
    bf16x4_t v;
    v[0] = (__bf16)a; v[1] = (__bf16)b; v[2] = (__bf16)c; v[3] = (__bf16)d;
    *reinterpret_cast<bf16x4_t*>(p) = v;
}

// ---- helpers of the one-workgroup backward kernel (heads of DH = 64 or 32 features) --------------------------
// The operands of a whole head are requested at once with direct-to-LDS loads, tile by tile, and a
// 64-row tile is consumed as soon as its own loads have landed: one memory latency per workgroup instead of one
// per tile.  LDS rows are dense (2 * DH bytes); the 16-byte chunk c of row r sits at position c ^ rsw<DH>(r), which
// serves both access patterns without padding: 16 consecutive rows of one chunk (operand fragments read row-wise)
// hit 16 distinct bank groups, and the rows of a transpose read spread evenly over the banks (128-byte rows: 8 rows x
// 64 B; 64-byte rows: 8 whole rows, contiguous).
template <int DH> __device__ __forceinline__ int rsw(int r);
template <> __device__ __forceinline__ int rsw<64>(int r) {
    const int p = (r >> 1) & 7;
    return ((p & 1) << 2) | (p >> 1);
}
template <> __device__ __forceinline__ int rsw<32>(int r) { return (r >> 2) & 3; }
// wavefront-wide load number i of a [nrows, ld] matrix with DH columns: rows RPL*i .. RPL*i + RPL-1 (RPL = 512 / DH
// rows of 2 * DH bytes, clamped to the last row) to the dense tile at dst
template <int DH>
__device__ __forceinline__ void res_dma8(unsigned char* dst, const bf16* __restrict__ base, int64_t ld, int nrows, int i, int lane) {
    constexpr int CPR = DH / 8, RPL = 64 / CPR;
    const int row = i * RPL + lane / CPR;
    const int c = (lane % CPR) ^ rsw<DH>(row);
    const unsigned voff = (unsigned)(min(row, nrows - 1) * (int)ld * 2 + c * 16);
    dma16_sbase(base, voff, (unsigned)(uintptr_t)LDS_PTR(unsigned char, dst) + i * 1024);
}
// Loads issued as inline assembly (the compiler's wait insertion neither sees them nor waits for the direct-to-LDS
// loads on their behalf); the caller waits with res_wait and then passes the registers through res_pin.
__device__ __forceinline__ u32x4_t res_load16(const void* p) {
    u32x4_t r;
    asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(r) : "v"(p) : "memory");
    return r;
}
__device__ __forceinline__ float res_load4(const void* p) {
    float r;
    asm volatile("global_load_dword %0, %1, off" : "=v"(r) : "v"(p) : "memory");
    return r;
}
// owned-row fragments of a head: lane (r = l%32, g) takes X[row0 + r][16*ks + 8g .. +7], rows clamped
template <int KS>
__device__ __forceinline__ void res_load_owned(const bf16* __restrict__ base, int64_t ld, int row0, int nrows, int lane,
                                               u32x4_t (&frag)[KS]) {
    const int r = min(row0 + (lane & 31), nrows - 1);
    const bf16* p = base + (int64_t)r * ld + 8 * (lane >> 5);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) frag[ks] = res_load16(p + 16 * ks);
}
__device__ __forceinline__ void res_pin(u32x4_t (&f)[4]) {
    asm volatile("" : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]));
}
__device__ __forceinline__ void res_pin(u32x4_t (&f)[2]) { asm volatile("" : "+v"(f[0]), "+v"(f[1])); }
__device__ __forceinline__ void res_pin(float& a) { asm volatile("" : "+v"(a)); }
template <int KS>
__device__ __forceinline__ void res_frags(const u32x4_t (&f)[KS], bf16x8_t (&b)[KS]) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) b[ks] = as_bf16x8(f[ks]);
}
// Requests rows [0, tp) of two matrices, 64-row tile by tile; returns through rem[j] how many of THIS wavefront's
// loads are younger than those of tile j (what may still be outstanding when tile j is consumed).
template <int DH>
__device__ __forceinline__ void res_request(unsigned char* d0, const bf16* b0, int64_t ld0, unsigned char* d1, const bf16* b1,
                                            int64_t ld1, int nrows, int tp, int wave, int nw, int lane, int (&rem)[4], int& total_out) {
    constexpr int RPL = 512 / DH, LPT = 64 / RPL;          // rows per wavefront-wide load, loads per 64-row tile
    int issued[4] = {0, 0, 0, 0}, total = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int i1 = min(LPT * j + LPT, tp / RPL);
        for (int i = LPT * j + wave; i < i1; i += nw) {
            res_dma8<DH>(d0, b0, ld0, nrows, i, lane);
            res_dma8<DH>(d1, b1, ld1, nrows, i, lane);
            total += 2;
        }
        issued[j] = total;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) rem[j] = total - issued[j];
    total_out = total;
}
// waits until at most n (wavefront-uniform, even, at most 16; anything else waits for all) vector-memory loads of the
// wavefront are outstanding
__device__ __forceinline__ void res_wait(int n) {
    switch (n) {
        case 0: __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0)); break;
        case 2: __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(2)); break;
        case 4: __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(4)); break;
        case 6: __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(6)); break;
        case 8: __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(8)); break;
        case 10: __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(10)); break;
        case 12: __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(12)); break;
        case 14: __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(14)); break;
        case 16: __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(16)); break;
        default: __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0)); break;
    }
}
// per-lane byte offsets of the two transpose reads of tr_frag<4, 8> in a resident tile, for r0 = 0 (any r0 that is a
// multiple of 16 adds r0 * 2 * DH) and feature tile dt
template <int DH>
__device__ __forceinline__ void res_tr_offsets(int lane, int dt, int& o1, int& o2) {
    const int j = lane & 15, q = lane >> 4;
    const int c = dt * 32 + (q & 1) * 16 + 4 * (j & 3);
    const int r = (q >> 1) * 4 + (j >> 2);
    o1 = r * (2 * DH) + (((c >> 3) ^ rsw<DH>(r)) << 4) + (c & 7) * 2;
    o2 = (r + 8) * (2 * DH) + (((c >> 3) ^ rsw<DH>(r + 8)) << 4) + (c & 7) * 2;
}
__device__ __forceinline__ bf16x8_t res_tr_frag(const unsigned char* tile_r0, int o1, int o2) {
    union { struct { s16x4_t lo, hi; } s; bf16x8_t v; } u;
    u.s.lo = lds_tr16(reinterpret_cast<const uint16_t*>(tile_r0 + o1));
    u.s.hi = lds_tr16(reinterpret_cast<const uint16_t*>(tile_r0 + o2));
    return u.v;
}

// ----------------------------------------------------------------------------------------
// forward
// ----------------------------------------------------------------------------------------
template <int DHP, bool PIPE>
__global__ __launch_bounds__(512) void attn_fwd_mfma(const bf16* __restrict__ qkv, bf16* __restrict__ o,
                                                     float* __restrict__ lse, const int* __restrict__ key_len,
                                                     int T, int H, int dh, int trows) {
    // trows: streamed rows held in LDS at a time -- 64, or all ceil32(T) rows when they fit (one load, no
    // further barriers)
    using C = AtCfg<DHP>;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    uint16_t* Ks0 = reinterpret_cast<uint16_t*>(smem);
    uint16_t* Vs0 = Ks0 + trows * C::PITCH;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    const int g = lane >> 5;
    const int bh = blockIdx.y, b = bh / H, h = bh % H;
    const int D = H * dh;
    const int64_t ld = 3 * (int64_t)D;
    const bf16* base = qkv + (int64_t)b * T * ld + h * dh;
    const int q0 = (blockIdx.x * nw + wave) * 32;
    // scores are kept in the base-2 domain (scale * log2 e folded into one multiply, exp2 is one instruction)
    const float c2 = rsqrtf((float)dh) * 1.4426950408889634f;
    // key-padding mask: keys at positions >= Tk take no part in the softmax (Tk = T without a mask)
    const int Tk = key_len ? min(max(key_len[b], 1), T) : T;

    bf16x8_t bq[C::KS];
    load_owned<DHP>(base, ld, q0, T, dh, lane, bq);

    f32x16_t accO[C::DT];
#pragma unroll
    for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) accO[dt][v] = 0.f;
    float m = -INFINITY, l = 0.f;

    // streamed mode (PIPE; trows == 64): the next 64-row tile is prefetched into registers during the products
    constexpr bool pipe = PIPE;
    TilePre<DHP> pk, pv;
    if constexpr (pipe) {
        tile_fetch<DHP>(pk, base + D, ld, 0, T, dh);
        tile_fetch<DHP>(pv, base + 2 * D, ld, 0, T, dh);
    }
    for (int t0 = 0; t0 < Tk; t0 += trows) {
      __syncthreads();
      if constexpr (pipe) {
          tile_store<DHP>(Ks0, pk);
          tile_store<DHP>(Vs0, pv);
      } else {
          load_tile<DHP>(Ks0, base + D, ld, t0, T, dh, trows);
          load_tile<DHP>(Vs0, base + 2 * D, ld, t0, T, dh, trows);
      }
      __syncthreads();
      if (pipe) if (t0 + trows < Tk) {
          tile_fetch<DHP>(pk, base + D, ld, t0 + trows, T, dh);
          tile_fetch<DHP>(pv, base + 2 * D, ld, t0 + trows, T, dh);
      }
      for (int k0 = t0; k0 < min(Tk, t0 + trows); k0 += AT_ROWS) {
        const uint16_t* Ks = Ks0 + (k0 - t0) * C::PITCH;
        const uint16_t* Vs = Vs0 + (k0 - t0) * C::PITCH;
        const int nt = (Tk - k0 > 32) ? 2 : 1;
        float s[2][16];
        float mloc = -INFINITY;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            if (t < nt) {
                f32x16_t acc;
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[v] = 0.f;
                const uint16_t* kp = Ks + (t * 32 + (lane & 31)) * C::PITCH + 8 * g;
#pragma unroll
                for (int ks = 0; ks < C::KS; ++ks)
                    acc = mfma32(*reinterpret_cast<const bf16x8_t*>(kp + 16 * ks), bq[ks], acc);
                if (k0 + t * 32 + 32 <= Tk) {               // whole tile inside the sequence: no masking
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        s[t][v] = acc[v] * c2;
                        mloc = fmaxf(mloc, s[t][v]);
                    }
                } else {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int key = k0 + t * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
                        s[t][v] = (key < Tk) ? acc[v] * c2 : -INFINITY;
                        mloc = fmaxf(mloc, s[t][v]);
                    }
                }
            }
        }
        mloc = fmaxf(mloc, __shfl_xor(mloc, 32, 64));
        const float mn = fmaxf(m, mloc);
        const float corr = __builtin_amdgcn_exp2f(m - mn);
        float lsum = 0.f;
#pragma unroll
        for (int t = 0; t < 2; ++t)
            if (t < nt) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    s[t][v] = __builtin_amdgcn_exp2f(s[t][v] - mn);
                    lsum += s[t][v];
                }
            }
        lsum += __shfl_xor(lsum, 32, 64);
        l = l * corr + lsum;
        m = mn;
#pragma unroll
        for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
            for (int v = 0; v < 16; ++v) accO[dt][v] *= corr;
#pragma unroll
        for (int t = 0; t < 2; ++t)
            if (t < nt) {
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    const bf16x8_t pb = pack8(&s[t][8 * c]);
#pragma unroll
                    for (int dt = 0; dt < C::DT; ++dt) {
                        const bf16x8_t a = tr_frag<4, 8>(Vs, C::PITCH, t * 32 + 16 * c, dt * 32, lane);
                        accO[dt] = mfma32(a, pb, accO[dt]);
                    }
                }
            }
      }
    }
    // O^T tile: lane holds query q0 + l%32, features dt*32 + 8*(v/4) + 4g + v%4
    const int q = q0 + (lane & 31);
    if (q < T) {
        const float inv = 1.f / l;
        bf16* orow = o + ((int64_t)b * T + q) * D + h * dh;
#pragma unroll
        for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                const int d = dt * 32 + 8 * v4 + 4 * g;
                if (d < dh)
                    store4_bf16(orow + d, accO[dt][4 * v4] * inv, accO[dt][4 * v4 + 1] * inv,
                                accO[dt][4 * v4 + 2] * inv, accO[dt][4 * v4 + 3] * inv);
            }
        if (g == 0) lse[(int64_t)bh * T + q] = (m + __log2f(l)) * 0.6931471805599453f;   // back to natural log
    }
}

// ----------------------------------------------------------------------------------------
// backward pass 1: dQ and delta (wavefront owns 32 query rows)
// ----------------------------------------------------------------------------------------
template <int DHP, bool PIPE>
__global__ __launch_bounds__(512) void attn_bwd_dq_mfma(const bf16* __restrict__ qkv, const bf16* __restrict__ o,
                                                        const bf16* __restrict__ dout, const float* __restrict__ lse,
                                                        bf16* __restrict__ dqkv, float* __restrict__ delta,
                                                        const int* __restrict__ key_len, int T, int H, int dh, int trows) {
    using C = AtCfg<DHP>;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    uint16_t* Ks0 = reinterpret_cast<uint16_t*>(smem);
    uint16_t* Vs0 = Ks0 + trows * C::PITCH;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    const int g = lane >> 5;
    const int bh = blockIdx.y, b = bh / H, h = bh % H;
    const int D = H * dh;
    const int64_t ld = 3 * (int64_t)D;
    const bf16* base = qkv + (int64_t)b * T * ld + h * dh;
    const bf16* dob = dout + (int64_t)b * T * D + h * dh;
    const bf16* ob = o + (int64_t)b * T * D + h * dh;
    const int q0 = (blockIdx.x * nw + wave) * 32;
    const int q = q0 + (lane & 31), qc = min(q, T - 1);
    const float scale = rsqrtf((float)dh);
    const float c2 = scale * 1.4426950408889634f;
    // key-padding mask: keys at positions >= Tk take no part in the softmax (Tk = T without a mask)
    const int Tk = key_len ? min(max(key_len[b], 1), T) : T;

    bf16x8_t bq[C::KS], bdo[C::KS];
    load_owned<DHP>(base, ld, q0, T, dh, lane, bq);
    load_owned<DHP>(dob, D, q0, T, dh, lane, bdo);
    // delta_q = sum_d dO[q,d] * O[q,d]; the two half-wavefronts hold complementary feature slots
    float dl = 0.f;
    {
        bf16x8_t bo[C::KS];
        load_owned<DHP>(ob, D, q0, T, dh, lane, bo);
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks)
#pragma unroll
            for (int e = 0; e < 8; ++e) dl += (float)bdo[ks][e] * (float)bo[ks][e];
        dl += __shfl_xor(dl, 32, 64);
    }
    const float L2 = lse[(int64_t)bh * T + qc] * 1.4426950408889634f;
    if (q < T && g == 0) delta[(int64_t)bh * T + q] = dl;

    f32x16_t accQ[C::DT];
#pragma unroll
    for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) accQ[dt][v] = 0.f;

    constexpr bool pipe = PIPE;
    TilePre<DHP> pk, pv;
    if constexpr (pipe) {
        tile_fetch<DHP>(pk, base + D, ld, 0, T, dh);
        tile_fetch<DHP>(pv, base + 2 * D, ld, 0, T, dh);
    }
    for (int t0 = 0; t0 < Tk; t0 += trows) {
      __syncthreads();
      if constexpr (pipe) {
          tile_store<DHP>(Ks0, pk);
          tile_store<DHP>(Vs0, pv);
      } else {
          load_tile<DHP>(Ks0, base + D, ld, t0, T, dh, trows);
          load_tile<DHP>(Vs0, base + 2 * D, ld, t0, T, dh, trows);
      }
      __syncthreads();
      if (pipe) if (t0 + trows < Tk) {
          tile_fetch<DHP>(pk, base + D, ld, t0 + trows, T, dh);
          tile_fetch<DHP>(pv, base + 2 * D, ld, t0 + trows, T, dh);
      }
      for (int k0 = t0; k0 < min(Tk, t0 + trows); k0 += AT_ROWS) {
        const uint16_t* Ks = Ks0 + (k0 - t0) * C::PITCH;
        const uint16_t* Vs = Vs0 + (k0 - t0) * C::PITCH;
        const int nt = (Tk - k0 > 32) ? 2 : 1;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            if (t < nt) {
                f32x16_t aS, aP;
#pragma unroll
                for (int v = 0; v < 16; ++v) { aS[v] = 0.f; aP[v] = 0.f; }
                const uint16_t* kp = Ks + (t * 32 + (lane & 31)) * C::PITCH + 8 * g;
                const uint16_t* vp = Vs + (t * 32 + (lane & 31)) * C::PITCH + 8 * g;
#pragma unroll
                for (int ks = 0; ks < C::KS; ++ks) {
                    aS = mfma32(*reinterpret_cast<const bf16x8_t*>(kp + 16 * ks), bq[ks], aS);
                    aP = mfma32(*reinterpret_cast<const bf16x8_t*>(vp + 16 * ks), bdo[ks], aP);
                }
                // dS without its 1/sqrt(head_dim): that factor is applied once to the finished dQ
                float ds[16];
                if (k0 + t * 32 + 32 <= Tk) {
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        ds[v] = __builtin_amdgcn_exp2f(aS[v] * c2 - L2) * (aP[v] - dl);
                } else {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int key = k0 + t * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
                        ds[v] = (key < Tk) ? __builtin_amdgcn_exp2f(aS[v] * c2 - L2) * (aP[v] - dl) : 0.f;
                    }
                }
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    const bf16x8_t dsb = pack8(&ds[8 * c]);
#pragma unroll
                    for (int dt = 0; dt < C::DT; ++dt) {
                        const bf16x8_t a = tr_frag<4, 8>(Ks, C::PITCH, t * 32 + 16 * c, dt * 32, lane);
                        accQ[dt] = mfma32(a, dsb, accQ[dt]);
                    }
                }
            }
        }
      }
    }
    if (q < T) {
        bf16* dq = dqkv + ((int64_t)b * T + q) * ld + h * dh;
#pragma unroll
        for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                const int d = dt * 32 + 8 * v4 + 4 * g;
                if (d < dh)
                    store4_bf16(dq + d, accQ[dt][4 * v4] * scale, accQ[dt][4 * v4 + 1] * scale,
                                accQ[dt][4 * v4 + 2] * scale, accQ[dt][4 * v4 + 3] * scale);
            }
    }
}

// ----------------------------------------------------------------------------------------
// backward pass 2: dK and dV (wavefront owns 32 key rows)
// ----------------------------------------------------------------------------------------
template <int DHP, bool PIPE>
__global__ __launch_bounds__(512) void attn_bwd_dkv_mfma(const bf16* __restrict__ qkv, const bf16* __restrict__ dout,
                                                         const float* __restrict__ lse, const float* __restrict__ delta,
                                                         bf16* __restrict__ dqkv, const int* __restrict__ key_len,
                                                         int T, int H, int dh, int trows) {
    using C = AtCfg<DHP>;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    uint16_t* Qs0 = reinterpret_cast<uint16_t*>(smem);
    uint16_t* Os0 = Qs0 + trows * C::PITCH;                       // dO tile
    float* lse_s0 = reinterpret_cast<float*>(Os0 + trows * C::PITCH);
    float* del_s0 = lse_s0 + trows;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    const int g = lane >> 5;
    const int bh = blockIdx.y, b = bh / H, h = bh % H;
    const int D = H * dh;
    const int64_t ld = 3 * (int64_t)D;
    const bf16* base = qkv + (int64_t)b * T * ld + h * dh;
    const bf16* dob = dout + (int64_t)b * T * D + h * dh;
    const int j0 = (blockIdx.x * nw + wave) * 32;
    const float scale = rsqrtf((float)dh);
    const float c2 = scale * 1.4426950408889634f;
    const int Tk = key_len ? min(max(key_len[b], 1), T) : T;      // keys beyond Tk are masked: their dK, dV are zero

    bf16x8_t bk[C::KS], bv[C::KS];
    load_owned<DHP>(base + D, ld, j0, T, dh, lane, bk);
    load_owned<DHP>(base + 2 * D, ld, j0, T, dh, lane, bv);

    f32x16_t accK[C::DT], accV[C::DT];
#pragma unroll
    for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) { accK[dt][v] = 0.f; accV[dt][v] = 0.f; }

    constexpr bool pipe = PIPE;
    TilePre<DHP> pq, po;
    float pre_l = 0.f, pre_d = 0.f;                                  // row statistics of the prefetched tile (thread r < 64: row r)
    auto stats_fetch = [&](int row0) {
        const int i = row0 + (int)threadIdx.x;
        if ((int)threadIdx.x < AT_ROWS) {
            pre_l = (i < T) ? lse[(int64_t)bh * T + i] * 1.4426950408889634f : INFINITY;
            pre_d = (i < T) ? delta[(int64_t)bh * T + i] : 0.f;
        }
    };
    if constexpr (pipe) {
        tile_fetch<DHP>(pq, base, ld, 0, T, dh);
        tile_fetch<DHP>(po, dob, D, 0, T, dh);
        stats_fetch(0);
    }
    for (int t0 = 0; t0 < T; t0 += trows) {
      __syncthreads();
      if constexpr (pipe) {
          tile_store<DHP>(Qs0, pq);
          tile_store<DHP>(Os0, po);
          if ((int)threadIdx.x < AT_ROWS) { lse_s0[threadIdx.x] = pre_l; del_s0[threadIdx.x] = pre_d; }
      } else {
          load_tile<DHP>(Qs0, base, ld, t0, T, dh, trows);
          load_tile<DHP>(Os0, dob, D, t0, T, dh, trows);
          for (int r = threadIdx.x; r < trows; r += blockDim.x) {
              const int i = t0 + r;
              // log-sum-exp in the base-2 domain; +inf masks rows beyond the sequence (exp2(. - inf) = 0)
              lse_s0[r] = (i < T) ? lse[(int64_t)bh * T + i] * 1.4426950408889634f : INFINITY;
              del_s0[r] = (i < T) ? delta[(int64_t)bh * T + i] : 0.f;
          }
      }
      __syncthreads();
      if (pipe) if (t0 + trows < T) {
          tile_fetch<DHP>(pq, base, ld, t0 + trows, T, dh);
          tile_fetch<DHP>(po, dob, D, t0 + trows, T, dh);
          stats_fetch(t0 + trows);
      }
      for (int i0 = t0; i0 < min(T, t0 + trows); i0 += AT_ROWS) {
        const uint16_t* Qs = Qs0 + (i0 - t0) * C::PITCH;
        const uint16_t* Os = Os0 + (i0 - t0) * C::PITCH;
        const float* lse_s = lse_s0 + (i0 - t0);
        const float* del_s = del_s0 + (i0 - t0);
        const int nt = (T - i0 > 32) ? 2 : 1;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            if (t < nt) {
                f32x16_t aS, aP;
#pragma unroll
                for (int v = 0; v < 16; ++v) { aS[v] = 0.f; aP[v] = 0.f; }
                const uint16_t* qp = Qs + (t * 32 + (lane & 31)) * C::PITCH + 8 * g;
                const uint16_t* op = Os + (t * 32 + (lane & 31)) * C::PITCH + 8 * g;
#pragma unroll
                for (int ks = 0; ks < C::KS; ++ks) {
                    aS = mfma32(*reinterpret_cast<const bf16x8_t*>(qp + 16 * ks), bk[ks], aS);
                    aP = mfma32(*reinterpret_cast<const bf16x8_t*>(op + 16 * ks), bv[ks], aP);
                }
                // lane: key j0 + l%32; rows i = i0 + t*32 + 8*(v/4) + 4g + v%4
                float p[16], ds[16];
#pragma unroll
                for (int v4 = 0; v4 < 4; ++v4) {
                    const int r = t * 32 + 8 * v4 + 4 * g;
                    const float4 Lr = *reinterpret_cast<const float4*>(lse_s + r);
                    const float4 Dr = *reinterpret_cast<const float4*>(del_s + r);
                    const float Lv[4] = {Lr.x, Lr.y, Lr.z, Lr.w};
                    const float Dv[4] = {Dr.x, Dr.y, Dr.z, Dr.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int v = 4 * v4 + e;
                        p[v] = __builtin_amdgcn_exp2f(aS[v] * c2 - Lv[e]);
                        ds[v] = p[v] * (aP[v] - Dv[e]);          // 1/sqrt(head_dim) applied to the finished dK
                    }
                }
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    const bf16x8_t pb = pack8(&p[8 * c]);
                    const bf16x8_t dsb = pack8(&ds[8 * c]);
#pragma unroll
                    for (int dt = 0; dt < C::DT; ++dt) {
                        const bf16x8_t ao = tr_frag<4, 8>(Os, C::PITCH, t * 32 + 16 * c, dt * 32, lane);
                        accV[dt] = mfma32(ao, pb, accV[dt]);
                        const bf16x8_t aq = tr_frag<4, 8>(Qs, C::PITCH, t * 32 + 16 * c, dt * 32, lane);
                        accK[dt] = mfma32(aq, dsb, accK[dt]);
                    }
                }
            }
        }
      }
    }
    const int j = j0 + (lane & 31);
    if (j >= Tk) {                       // a masked key: no query looked at it
#pragma unroll
        for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
            for (int v = 0; v < 16; ++v) { accK[dt][v] = 0.f; accV[dt][v] = 0.f; }
    }
    if (j < T) {
        bf16* dk = dqkv + ((int64_t)b * T + j) * ld + D + h * dh;
        bf16* dv = dk + D;
#pragma unroll
        for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                const int d = dt * 32 + 8 * v4 + 4 * g;
                if (d < dh) {
                    store4_bf16(dk + d, accK[dt][4 * v4] * scale, accK[dt][4 * v4 + 1] * scale,
                                accK[dt][4 * v4 + 2] * scale, accK[dt][4 * v4 + 3] * scale);
                    store4_bf16(dv + d, accV[dt][4 * v4], accV[dt][4 * v4 + 1], accV[dt][4 * v4 + 2], accV[dt][4 * v4 + 3]);
                }
            }
    }
}

#define RES_BARRIER(n) do { asm volatile("" ::: "memory"); res_wait(n); __builtin_amdgcn_s_barrier(); asm volatile("" ::: "memory"); } while (0)

// ----------------------------------------------------------------------------------------
// backward, both passes in one workgroup per head (heads of DH = 64 or 32 features, up to 256 tokens): Q, K, V and dO of the head
// are brought to LDS once; every wavefront first runs pass 1 for its 32 query rows (dQ, delta), then, after one
// barrier, pass 2 for its 32 key rows (dK, dV) with the row statistics of pass 1 read from LDS.  Same arithmetic, in
// the same order, as the two separate kernels; half their memory traffic.
// ----------------------------------------------------------------------------------------
template <int DH>
__global__ __launch_bounds__(512) void attn_bwd_fused(const bf16* __restrict__ qkv, const bf16* __restrict__ o,
                                                        const bf16* __restrict__ dout, const float* __restrict__ lse,
                                                        bf16* __restrict__ dqkv, float* __restrict__ delta,
                                                        const int* __restrict__ key_len, int T, int H) {
    constexpr int KS = DH / 16, DT = DH / 32, dh = DH, ROWB = 2 * DH;
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    const int tp = (T + 31) / 32 * 32;               // == 32 * wavefronts of the workgroup
    unsigned char* Ks0 = smem;
    unsigned char* Vs0 = Ks0 + tp * ROWB;
    unsigned char* Qs0 = Vs0 + tp * ROWB;
    unsigned char* Os0 = Qs0 + tp * ROWB;             // dO
    float* lse_s0 = reinterpret_cast<float*>(Os0 + tp * ROWB);
    float* del_s0 = lse_s0 + tp;
    const int lane = threadIdx.x & 63, nw = blockDim.x >> 6;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane >> 5;
    const int bh = blockIdx.x, b = bh / H, h = bh % H;
    const int D = H * dh;
    const int64_t ld = 3 * (int64_t)D;
    const bf16* base = qkv + (int64_t)b * T * ld + h * dh;
    const bf16* dob = dout + (int64_t)b * T * D + h * dh;
    const bf16* ob = o + (int64_t)b * T * D + h * dh;
    const int r0 = wave * 32;                        // this wavefront's query rows (pass 1) and key rows (pass 2)
    const int q = r0 + (lane & 31), qc = min(q, T - 1);
    const float scale = rsqrtf((float)dh);
    const float c2 = scale * 1.4426950408889634f;
    const int Tk = key_len ? min(max(key_len[b], 1), T) : T;
    // ---- requests: owned rows of pass 1 to registers, then K and V (tile by tile), then Q and dO ----
    u32x4_t fq[KS], fdo[KS], fo[KS];
    res_load_owned<KS>(base, ld, r0, T, lane, fq);
    res_load_owned<KS>(dob, D, r0, T, lane, fdo);
    res_load_owned<KS>(ob, D, r0, T, lane, fo);
    float Lraw = res_load4(lse + (int64_t)bh * T + qc);
    int rem[4], nkv, nqo;
    res_request<DH>(Ks0, base + D, ld, Vs0, base + 2 * D, ld, T, tp, wave, nw, lane, rem, nkv);
    {
        int rem2[4];
        res_request<DH>(Qs0, base, ld, Os0, dob, D, T, tp, wave, nw, lane, rem2, nqo);
    }
    res_wait(min(nkv + nqo, 16));                    // the owned rows are older than every direct-to-LDS load
    res_pin(fq); res_pin(fdo); res_pin(fo); res_pin(Lraw);

    int rowoff[KS], o1[DT], o2[DT];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) rowoff[ks] = (lane & 31) * ROWB + (((2 * ks + g) ^ rsw<DH>(lane & 31)) << 4);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) res_tr_offsets<DH>(lane, dt, o1[dt], o2[dt]);

    // ---- pass 1: dQ, delta ----
    {
        bf16x8_t bq[KS], bdo[KS], bo[KS];
        res_frags<KS>(fq, bq); res_frags<KS>(fdo, bdo); res_frags<KS>(fo, bo);
        const float L2 = Lraw * 1.4426950408889634f;
        float dl = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int e = 0; e < 8; ++e) dl += (float)bdo[ks][e] * (float)bo[ks][e];
        dl += __shfl_xor(dl, 32, 64);
        if (g == 0) {
            if (q < T) delta[(int64_t)bh * T + q] = dl;
            // statistics for pass 2; +inf masks rows beyond the sequence (exp2(. - inf) = 0)
            lse_s0[q] = (q < T) ? L2 : INFINITY;
            del_s0[q] = (q < T) ? dl : 0.f;
        }

        f32x16_t accQ[DT];
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int v = 0; v < 16; ++v) accQ[dt][v] = 0.f;

#pragma unroll
        for (int jt = 0; jt < 4; ++jt) {
            const int k0 = jt * 64;
            if (k0 < Tk) {
            RES_BARRIER(min(rem[jt] + nqo, 16));
            const unsigned char* Ks = Ks0 + k0 * ROWB;
            const unsigned char* Vs = Vs0 + k0 * ROWB;
            const int nt = (Tk - k0 > 32) ? 2 : 1;
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                if (t < nt) {
                    f32x16_t aS, aP;
#pragma unroll
                    for (int v = 0; v < 16; ++v) { aS[v] = 0.f; aP[v] = 0.f; }
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) {
                        aS = mfma32(*reinterpret_cast<const bf16x8_t*>(Ks + t * 32 * ROWB + rowoff[ks]), bq[ks], aS);
                        aP = mfma32(*reinterpret_cast<const bf16x8_t*>(Vs + t * 32 * ROWB + rowoff[ks]), bdo[ks], aP);
                    }
                    float ds[16];
                    if (k0 + t * 32 + 32 <= Tk) {
#pragma unroll
                        for (int v = 0; v < 16; ++v)
                            ds[v] = __builtin_amdgcn_exp2f(aS[v] * c2 - L2) * (aP[v] - dl);
                    } else {
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const int key = k0 + t * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
                            ds[v] = (key < Tk) ? __builtin_amdgcn_exp2f(aS[v] * c2 - L2) * (aP[v] - dl) : 0.f;
                        }
                    }
#pragma unroll
                    for (int c = 0; c < 2; ++c) {
                        const bf16x8_t dsb = pack8(&ds[8 * c]);
#pragma unroll
                        for (int dt = 0; dt < DT; ++dt) {
                            const bf16x8_t a = res_tr_frag(Ks + (t * 32 + 16 * c) * ROWB, o1[dt], o2[dt]);
                            accQ[dt] = mfma32(a, dsb, accQ[dt]);
                        }
                    }
                }
            }
            }
        }
        if (q < T) {
            bf16* dq = dqkv + ((int64_t)b * T + q) * ld + h * dh;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int v4 = 0; v4 < 4; ++v4) {
                    const int d = dt * 32 + 8 * v4 + 4 * g;
                    store4_bf16(dq + d, accQ[dt][4 * v4] * scale, accQ[dt][4 * v4 + 1] * scale,
                                accQ[dt][4 * v4 + 2] * scale, accQ[dt][4 * v4 + 3] * scale);
                }
        }
    }
    // ---- every load has landed, every wavefront has left its statistics ----
    RES_BARRIER(0);

    // ---- pass 2: dK, dV ----
    {
        bf16x8_t bk[KS], bv[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            bk[ks] = *reinterpret_cast<const bf16x8_t*>(Ks0 + r0 * ROWB + rowoff[ks]);
            bv[ks] = *reinterpret_cast<const bf16x8_t*>(Vs0 + r0 * ROWB + rowoff[ks]);
        }
        f32x16_t accK[DT], accV[DT];
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int v = 0; v < 16; ++v) { accK[dt][v] = 0.f; accV[dt][v] = 0.f; }

        for (int i0 = 0; i0 < T; i0 += 64) {
            const unsigned char* Qs = Qs0 + i0 * ROWB;
            const unsigned char* Os = Os0 + i0 * ROWB;
            const float* lse_s = lse_s0 + i0;
            const float* del_s = del_s0 + i0;
            const int nt = (T - i0 > 32) ? 2 : 1;
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                if (t < nt) {
                    f32x16_t aS, aP;
#pragma unroll
                    for (int v = 0; v < 16; ++v) { aS[v] = 0.f; aP[v] = 0.f; }
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) {
                        aS = mfma32(*reinterpret_cast<const bf16x8_t*>(Qs + t * 32 * ROWB + rowoff[ks]), bk[ks], aS);
                        aP = mfma32(*reinterpret_cast<const bf16x8_t*>(Os + t * 32 * ROWB + rowoff[ks]), bv[ks], aP);
                    }
                    float p[16], ds[16];
#pragma unroll
                    for (int v4 = 0; v4 < 4; ++v4) {
                        const int r = t * 32 + 8 * v4 + 4 * g;
                        const float4 Lr = *reinterpret_cast<const float4*>(lse_s + r);
                        const float4 Dr = *reinterpret_cast<const float4*>(del_s + r);
                        const float Lv[4] = {Lr.x, Lr.y, Lr.z, Lr.w};
                        const float Dv[4] = {Dr.x, Dr.y, Dr.z, Dr.w};
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const int v = 4 * v4 + e;
                            p[v] = __builtin_amdgcn_exp2f(aS[v] * c2 - Lv[e]);
                            ds[v] = p[v] * (aP[v] - Dv[e]);
                        }
                    }
#pragma unroll
                    for (int c = 0; c < 2; ++c) {
                        const bf16x8_t pb = pack8(&p[8 * c]);
                        const bf16x8_t dsb = pack8(&ds[8 * c]);
#pragma unroll
                        for (int dt = 0; dt < DT; ++dt) {
                            const bf16x8_t ao = res_tr_frag(Os + (t * 32 + 16 * c) * ROWB, o1[dt], o2[dt]);
                            accV[dt] = mfma32(ao, pb, accV[dt]);
                            const bf16x8_t aq = res_tr_frag(Qs + (t * 32 + 16 * c) * ROWB, o1[dt], o2[dt]);
                            accK[dt] = mfma32(aq, dsb, accK[dt]);
                        }
                    }
                }
            }
        }
        const int j = r0 + (lane & 31);
        if (j >= Tk) {
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int v = 0; v < 16; ++v) { accK[dt][v] = 0.f; accV[dt][v] = 0.f; }
        }
        if (j < T) {
            bf16* dk = dqkv + ((int64_t)b * T + j) * ld + D + h * dh;
            bf16* dv = dk + D;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int v4 = 0; v4 < 4; ++v4) {
                    const int d = dt * 32 + 8 * v4 + 4 * g;
                    store4_bf16(dk + d, accK[dt][4 * v4] * scale, accK[dt][4 * v4 + 1] * scale,
                                accK[dt][4 * v4 + 2] * scale, accK[dt][4 * v4 + 3] * scale);
                    store4_bf16(dv + d, accV[dt][4 * v4], accV[dt][4 * v4 + 1], accV[dt][4 * v4 + 2], accV[dt][4 * v4 + 3]);
                }
        }
    }
}

// ----------------------------------------------------------------------------------------
// launchers
// ----------------------------------------------------------------------------------------
// Wavefronts per workgroup: split the ceil(T/32) row tiles evenly over as few workgroups as
// 8 wavefronts each allow (T=197: 1 x 7, T=257: 2 x 5, T=512: 2 x 8).
#define RC_LDS(expr) do { int _rc = (expr); if (_rc != REV_OK) return _rc; } while (0)

static void row_split(int T, int* nblk, int* nw) {
    const int tiles = (T + 31) / 32;
    *nblk = (tiles + 7) / 8;
    *nw = (tiles + *nblk - 1) / *nblk;
}

// Rows of the streamed operands kept in LDS at a time: every (32-padded) row of the head when two such
// tiles plus the row statistics fit in 128 KB -- then a workgroup loads once and never synchronises
// again (measured faster than streaming even where only one such workgroup fits a CU: 257 tokens at
// head_dim 80) -- otherwise 64-row tiles.
template <int DHP>
static int tile_rows(int T) {
    const int all = (T + 31) / 32 * 32;
    const size_t bytes = (size_t)2 * all * AtCfg<DHP>::PITCH * sizeof(uint16_t) + 2 * all * sizeof(float);
    return bytes <= 128 * 1024 ? all : AT_ROWS;
}

template <typename K>
static int raise_lds(K kern, size_t shmem) {
    if (shmem > 64 * 1024)
        REV_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
    return REV_OK;
}

template <int DHP>
static int fwd_launch(hipStream_t s, const bf16* qkv, bf16* o, float* lse, int B, int T, int H, int dh, const int* key_len) {
    int nblk, nw;
    row_split(T, &nblk, &nw);
    const int trows = tile_rows<DHP>(T);
    const size_t shmem = (size_t)2 * trows * AtCfg<DHP>::PITCH * sizeof(uint16_t);
    // (the register prefetch of the streamed mode costs the forward kernel one resident wavefront per
    // SIMD and measured slower there; the backward kernels gain 20 % from it)
    RC_LDS(raise_lds(attn_fwd_mfma<DHP, false>, shmem));
    hipLaunchKernelGGL((attn_fwd_mfma<DHP, false>), dim3(nblk, B * H), dim3(nw * 64), shmem, s, qkv, o, lse, key_len, T, H, dh, trows);
    REV_HIP(hipGetLastError());
    return REV_OK;
}

template <int DHP>
static int bwd_launch(hipStream_t s, const bf16* qkv, const bf16* o, const bf16* dout, const float* lse, bf16* dqkv,
                      float* delta, int B, int T, int H, int dh, const int* key_len, bool solo) {
    // Heads of 64 or 32 features and up to 256 tokens: one workgroup per head runs both passes from one LDS copy of
    // the head (14-20 % faster than the two kernels at 197 tokens, 40 % at 49; same arithmetic in the same order, so
    // the same bits).  Under both schedules: A/B on two boxes, the parallel schedule gains 3.7 % from it on Rev-ViT-B
    // and 4.6 % on Rev-ViT-S, the sequential one 1.5 %.
    if constexpr (DHP == 64 || DHP == 32) {
        if (dh == DHP && T <= 256) {
            const int tiles = (T + 31) / 32;
            const size_t shmem = (size_t)tiles * 32 * (4 * 2 * DHP + 8);
            RC_LDS(raise_lds(attn_bwd_fused<DHP>, shmem));
            hipLaunchKernelGGL(attn_bwd_fused<DHP>, dim3(B * H), dim3(tiles * 64), shmem, s, qkv, o, dout, lse, dqkv, delta, key_len, T, H);
            REV_HIP(hipGetLastError());
            return REV_OK;
        }
    }
    int nblk, nw;
    row_split(T, &nblk, &nw);
    // A head's row tiles are split over 4-wavefront workgroups: the backward kernels need 160-210 registers, so only
    // one 5...8-wavefront workgroup fits a CU but three (two) of 4 wavefronts do -- 4 % (197 tokens) to 12 % (257
    // tokens) faster alone.  Next to another stream's kernels the extra resident workgroups cost the neighbour; measured
    // in the parallel schedule: 257 tokens (9 row tiles) +1.9 % with the split, 512 tokens (16 row tiles) -0.7 %, so
    // there it is taken up to 12 row tiles.  A wavefront's work does not depend on the grouping, so the results are
    // bit-identical.
    if ((solo || (T + 31) / 32 <= 12) && nw > 4) {
        nblk = ((T + 31) / 32 + 3) / 4;
        nw = 4;
    }
    // With 4 or more wavefronts the backward kernels always stream 64-row tiles with the next tile
    // prefetched into registers: measured 6-8 % faster than keeping the head resident (197 and 257
    // tokens), with a fifth of the LDS, which also leaves room for a co-running kernel of the other stream.
    const int trows = (nw >= 4) ? AT_ROWS : tile_rows<DHP>(T);
    const size_t shmem = (size_t)2 * trows * AtCfg<DHP>::PITCH * sizeof(uint16_t);
    const size_t shmem2 = shmem + 2 * trows * sizeof(float);
    if (trows == AT_ROWS && nw >= 4) {          // streamed mode with register prefetch of the next tile
        hipLaunchKernelGGL((attn_bwd_dq_mfma<DHP, true>), dim3(nblk, B * H), dim3(nw * 64), shmem, s, qkv, o, dout, lse, dqkv,
                           delta, key_len, T, H, dh, trows);
        hipLaunchKernelGGL((attn_bwd_dkv_mfma<DHP, true>), dim3(nblk, B * H), dim3(nw * 64), shmem2, s, qkv, dout, lse, delta,
                           dqkv, key_len, T, H, dh, trows);
    } else {
        RC_LDS(raise_lds(attn_bwd_dq_mfma<DHP, false>, shmem));
        RC_LDS(raise_lds(attn_bwd_dkv_mfma<DHP, false>, shmem2));
        hipLaunchKernelGGL((attn_bwd_dq_mfma<DHP, false>), dim3(nblk, B * H), dim3(nw * 64), shmem, s, qkv, o, dout, lse, dqkv,
                           delta, key_len, T, H, dh, trows);
        hipLaunchKernelGGL((attn_bwd_dkv_mfma<DHP, false>), dim3(nblk, B * H), dim3(nw * 64), shmem2, s, qkv, dout, lse, delta,
                           dqkv, key_len, T, H, dh, trows);
    }
    REV_HIP(hipGetLastError());
    return REV_OK;
}

static bool mfma_ok(const void* a, const void* b, const void* c, const void* d) {
    return (((uintptr_t)a | (uintptr_t)b | (uintptr_t)c | (uintptr_t)d) & 15) == 0;
}

template <>
int attention_forward<bf16>(hipStream_t s, const bf16* qkv, bf16* o, float* lse, int B, int T, int H, int dh, const int* key_len) {
    if ((dh & 7) || dh > 128 || !mfma_ok(qkv, o, nullptr, nullptr))
        return attention_forward_simple<bf16>(s, qkv, o, lse, B, T, H, dh, key_len);
    ProfScope ps(K_ATTN_FWD, s, 4.0 * B * H * (double)T * T * dh);
    if (dh <= 32) return fwd_launch<32>(s, qkv, o, lse, B, T, H, dh, key_len);
    if (dh <= 64) return fwd_launch<64>(s, qkv, o, lse, B, T, H, dh, key_len);
    if (dh <= 96) return fwd_launch<96>(s, qkv, o, lse, B, T, H, dh, key_len);
    return fwd_launch<128>(s, qkv, o, lse, B, T, H, dh, key_len);
}
template <>
int attention_forward<float>(hipStream_t s, const float* qkv, float* o, float* lse, int B, int T, int H, int dh, const int* key_len) {
    return attention_forward_simple<float>(s, qkv, o, lse, B, T, H, dh, key_len);
}

template <>
int attention_backward<bf16>(hipStream_t s, const bf16* qkv, const bf16* o, const bf16* dout, const float* lse,
                             bf16* dqkv, float* delta, int B, int T, int H, int dh, const int* key_len, bool solo) {
    // Heads wider than 96 take the plain-ALU kernels: the matrix-core dK/dV kernel would need more registers
    // than a wavefront has for a 128-wide head (it spilled), and no workload of the path has such heads.
    if ((dh & 7) || dh > 96 || !mfma_ok(qkv, o, dout, dqkv))
        return attention_backward_simple<bf16>(s, qkv, o, dout, lse, dqkv, delta, B, T, H, dh, key_len);
    ProfScope ps(K_ATTN_BWD, s, 8.0 * B * H * (double)T * T * dh);
    if (dh <= 32) return bwd_launch<32>(s, qkv, o, dout, lse, dqkv, delta, B, T, H, dh, key_len, solo);
    if (dh <= 64) return bwd_launch<64>(s, qkv, o, dout, lse, dqkv, delta, B, T, H, dh, key_len, solo);
    return bwd_launch<96>(s, qkv, o, dout, lse, dqkv, delta, B, T, H, dh, key_len, solo);
}
template <>
int attention_backward<float>(hipStream_t s, const float* qkv, const float* o, const float* dout, const float* lse,
                              float* dqkv, float* delta, int B, int T, int H, int dh, const int* key_len, bool) {
    return attention_backward_simple<float>(s, qkv, o, dout, lse, dqkv, delta, B, T, H, dh, key_len);
}

}  // namespace rev
