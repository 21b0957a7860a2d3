// Device helpers shared by the MFMA kernels (gfx950 only).
#pragma once
#include "common.h"

namespace unigist {

typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

// ---------------------------------------------------------------------------------------------
// Tiles staged with direct global->LDS loads (global_load_lds_dwordx4).
// One such instruction makes a wave write 64 x 16 B = 1 KB of consecutive LDS, so rows cannot be
// padded; bank conflicts are avoided by permuting the 16-byte chunks of each row instead (swz16 below).
// CH = chunks per row (D / 8).

// issue one 1 KB direct load: lane `lane` fetches 16 bytes from `src` into lds_base + 16 * lane
__device__ __forceinline__ void g2l16(const void* src, void* lds_base_uniform) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                     (__attribute__((address_space(3))) void*)lds_base_uniform, 16, 0, 0);
}

// wait until this wave's outstanding vector-memory operations (direct loads included) are done
__device__ __forceinline__ void wait_vmem() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// ---------------------------------------------------------------------------------------------
// v_mfma_f32_16x16x32_bf16 (D = A * B + C, A 16 x 32, B 32 x 16).  With r16 = lane % 16 and g4 = lane / 16:
//   A: lane holds A[r16][8 g4 .. 8 g4 + 7]      B: lane holds B[8 g4 .. 8 g4 + 7][r16]
//   C/D: register i holds D[4 g4 + i][r16]
// The C registers of two 16-row blocks kb = 0, 1, read as a B operand, stand for the contraction slots
// 8 g4 + 4 kb + i = row 16 kb + 4 g4 + i; tr16_frag16() fetches the matching A operand from a row-major tile.
__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x4 zero4() { return f32x4{0.f, 0.f, 0.f, 0.f}; }

// a * b for factors below 2^24 on the full-rate 24-bit multiplier (the compiler picks the quarter-rate 32-bit one).
__device__ __forceinline__ int mul24(int a, int b) {
    int r;
    asm("v_mul_u32_u24 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

// Chunk swizzle for tiles read in that shape: chunk ch of tile row r is stored at chunk position ch ^ swz16(r).
// Its period of 16 rows puts the 16 rows of a row-wise fragment read and the 4 rows of a transposing read on
// distinct banks; the two transposing reads of a fragment lie 16 rows apart and so share one address register.
template <int CH>
__device__ __forceinline__ int swz16(int r) { return CH == 16 ? (r & 15) : ((r >> 1) & 7); }

// byte offset, inside a tile swizzled with swz16, of the row-wise fragment chunk of this lane: row r16, chunk 4 ks + g4
template <int CH>
__device__ __forceinline__ int row16_lane_off(int ks) {
    const int lane = threadIdx.x & 63, r16 = lane & 15, g4 = lane >> 4;
    return r16 * (CH * 16) + (((4 * ks + g4) ^ swz16<CH>(r16)) << 4);
}
// ... and of this lane's piece of the transposing read of the 4 x 16 block rows 4 g4 .. +3, columns 16 db .. +15:
// lane p of a 16-lane group passes the address of X[4 g4 + p/4][16 db + 4 (p%4)] and receives X[4 g4 .. +3][16 db + p]
template <int CH>
__device__ __forceinline__ int tr16_lane_off16(int db) {
    const int lane = threadIdx.x & 63, r16 = lane & 15, g4 = lane >> 4;
    const int rl = 4 * g4 + (r16 >> 2);
    const int ch = 2 * db + ((r16 & 3) >> 1);
    return rl * (CH * 16) + ((ch ^ swz16<CH>(rl)) << 4) + (r16 & 1) * 8;
}
// A operand X^T for 32 contraction rows starting at row0 (a multiple of 16), 16-column block fixed by the lane offset
template <int CH>
__device__ __forceinline__ bf16x8 tr16_frag16(const char* tile_plus_lane_off, int row0) {
    const char* a = tile_plus_lane_off + row0 * (CH * 16);
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)a);
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(a + 16 * CH * 16));
    s16x8 r = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, r);
}
// two C register quads (blocks kb = 0, 1) -> bf16 B operand
__device__ __forceinline__ bf16x8 pack44(const f32x4& x0, const f32x4& x1) {
    u32x4 r;
    r[0] = pack_bf16x2(x0[0], x0[1]);
    r[1] = pack_bf16x2(x0[2], x0[3]);
    r[2] = pack_bf16x2(x1[0], x1[1]);
    r[3] = pack_bf16x2(x1[2], x1[3]);
    return __builtin_bit_cast(bf16x8, r);
}

}  // namespace unigist
