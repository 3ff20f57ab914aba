// Matrix-core and LDS helpers shared by the bf16 GEMM and attention kernels (gfx950).
//
// v_mfma_f32_32x32x16_bf16, per lane l of the wavefront (g = l / 32):
//   A operand: row l%32, contraction slots 8g .. 8g+7;  B operand: column l%32, same slots;
//   D: column l%32, rows 8*(v/4) + 4g + v%4 for accumulator register v = 0..15.
// The contraction slots may stand for any 16 indices as long as A and B agree.
#pragma once
#include "common.h"

namespace rev {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

__device__ __forceinline__ f32x16_t mfma32(bf16x8_t a, bf16x8_t b, f32x16_t c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// LDS transpose read (ds_read_b64_tr_b16): the 16 lanes of a group hand in a 4x4
// arrangement of 8-byte chunks (lane 4e+q: row e, columns 4q..4q+3 of a 4x16 patch)
// and lane j of the group receives column j of the patch: 4 consecutive rows.
__device__ __forceinline__ s16x4_t lds_tr16(const uint16_t* p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4_t, p));
}

// Operand fragment for 32 columns c0..c0+31 of a row-major LDS tile whose ROWS are
// the contraction index.  Lane (l%32, g) receives rows  r0 + GS*g + {0..3}  and
// r0 + GS*g + SEC + {0..3}  of column c0 + l%32.
//   GS = 8, SEC = 4: slots are 16 consecutive rows r0..r0+15;
//   GS = 4, SEC = 8: slots follow the accumulator row order {4g..4g+3, 8+4g..8+4g+3},
//                    so a D tile converted in place can be the other operand.
template <int GS, int SEC>
__device__ __forceinline__ bf16x8_t tr_frag(const uint16_t* tile, int pitch, int r0, int c0, int lane) {
    const int j = lane & 15, q = lane >> 4;
    const int c = c0 + (q & 1) * 16 + 4 * (j & 3);
    const int r = r0 + (q >> 1) * GS + (j >> 2);
    const uint16_t* p = tile + r * pitch + c;
    union { struct { s16x4_t lo, hi; } s; bf16x8_t v; } u;
    u.s.lo = lds_tr16(p);
    u.s.hi = lds_tr16(p + SEC * pitch);
    return u.v;
}

// Same fragment from a DENSE tile with 256-byte rows (128 bf16) whose 16-byte chunk c of row r
// sits at position c ^ (4 * (r & 3)) -- the layout a direct-to-LDS load can produce.  One transpose
// read touches 4 consecutive rows x 64 bytes per 32 lanes; the swizzle spreads the 4 rows over the
// 4 quarters of the bank space.  Slots: the 16 consecutive rows r0..r0+15 (r0 a multiple of 4).
__device__ __forceinline__ bf16x8_t tr_frag_swz(const unsigned char* tile, int r0, int c0, int lane) {
    const int j = lane & 15, q = lane >> 4;
    const int c = c0 + (q & 1) * 16 + 4 * (j & 3);       // first of 4 columns
    const int r = r0 + (q >> 1) * 8 + (j >> 2);          // r & 3 == (j >> 2) & 3
    const int pos = (c >> 3) ^ (4 * (r & 3));
    const unsigned char* p = tile + r * 256 + pos * 16 + (c & 7) * 2;
    union { struct { s16x4_t lo, hi; } s; bf16x8_t v; } u;
    u.s.lo = lds_tr16(reinterpret_cast<const uint16_t*>(p));
    u.s.hi = lds_tr16(reinterpret_cast<const uint16_t*>(p + 4 * 256));   // rows +4: same r & 3
    return u.v;
}

// ---- hand-placed LDS fragment reads -------------------------------------------------------------
// The compiler waits for ALL outstanding LDS reads (lgkmcnt(0)) before the first product that uses
// any of them, which serialises the read latency with the matrix-core work twice per stage.  The
// reads below are therefore issued as inline assembly, all of a stage's groups up front (or two
// groups ahead), and every product group waits only for its own operands: LDS reads return in
// order, so "at most n still outstanding" means the oldest ones have landed.  The wait statements
// carry the fragment registers as read-write operands, which pins the products behind them.
__device__ __forceinline__ u32x4_t lds_read_b128(unsigned addr, int imm) {
    u32x4_t r;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(imm) : "memory");
    return r;
}
__device__ __forceinline__ u32x2_t lds_read_tr16_b64(unsigned addr, int imm) {
    u32x2_t r;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(imm) : "memory");
    return r;
}
template <int N>
__device__ __forceinline__ void lds_wait4(u32x4_t& a0, u32x4_t& a1, u32x4_t& b0, u32x4_t& b1) {
    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(a0), "+v"(a1), "+v"(b0), "+v"(b1) : "n"(N));
}
template <int N>
__device__ __forceinline__ void lds_wait7(u32x4_t& a0, u32x4_t& a1, u32x4_t& a2, u32x4_t& a3, u32x4_t& a4, u32x4_t& b0,
                                          u32x4_t& b1) {
    asm volatile("s_waitcnt lgkmcnt(%7)" : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4), "+v"(b0), "+v"(b1) : "n"(N));
}
__device__ __forceinline__ bf16x8_t as_bf16x8(u32x4_t v) { return __builtin_bit_cast(bf16x8_t, v); }
__device__ __forceinline__ u32x4_t join64(u32x2_t lo, u32x2_t hi) { return u32x4_t{lo[0], lo[1], hi[0], hi[1]}; }

// Direct-to-LDS load of 16 bytes per lane in the scalar-base form: global address = sbase + voff
// (per-lane 32-bit byte offset), LDS destination = lds_addr (wavefront-uniform) + 16 * lane.
// Written out because the compiler otherwise rebuilds 64-bit per-lane pointers inside loops.
__device__ __forceinline__ void dma16_sbase(const void* sbase, unsigned voff, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(voff), "s"(sbase), "s"(lds_addr) : "memory", "m0");
}

// 64 bytes of zeros (never written): the source of direct-to-LDS loads that fall outside a matrix
static __device__ u32x4_t g_zero_chunk[4];

#define GLB_PTR(p) ((__attribute__((address_space(1))) const void*)(p))
// s_waitcnt immediate for gfx9: vmcnt in bits [3:0] and [15:14], expcnt [6:4] (no wait), lgkmcnt [11:8] = 0
constexpr int waitcnt_vm_lgkm0(int vm) { return (vm & 15) | ((vm >> 4) << 14) | (7 << 4); }

// Workgroups go round-robin over the 8 XCDs, each with its own L2: give every
// XCD one contiguous run of tiles so that neighbouring tiles (which share an
// operand panel) meet in the same L2.
__device__ __forceinline__ int xcd_remap(int b, int nblk) {
    const int per = nblk >> 3;
    if (b >= per * 8) return b;
    return (b & 7) * per + (b >> 3);
}

}  // namespace rev
