// Device helpers shared by the MFMA kernels (gfx950 only).
//
// Fragment layouts of v_mfma_f32_32x32x16_bf16 (D = A * B + C, A is 32 x 16, B is 16 x 32), with
// c32 = lane % 32 and h = lane / 32:
//   A: lane holds A[c32][8h .. 8h+7]          B: lane holds B[8h .. 8h+7][c32]
//   C/D: register i holds D[8 (i/4) + 4h + i%4][c32]
// Since the contraction index can be permuted freely as long as A and B agree, the 8 C registers
// 8t .. 8t+7 of a lane, read as a B operand, stand for the contraction slots (8 (2t) + 4h + 0..3) and
// (8 (2t+1) + 4h + 0..3); tr16_frag() below fetches the matching A operand from a row-major tile.
#pragma once
#include "common.h"

namespace unigist {

typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ f32x16 zero16() {
    f32x16 z;
#pragma unroll
    for (int i = 0; i < 16; ++i) z[i] = 0.f;
    return z;
}

// value held by lane ^ 32
__device__ __forceinline__ float other_half(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(unsigned, x), __builtin_bit_cast(unsigned, x), false,
                                              false);
    // lanes < 32 find the partner's value in r[1], lanes >= 32 in r[0]; the other slot is their own
    float a = __builtin_bit_cast(float, (unsigned)r[0]);
    float b = __builtin_bit_cast(float, (unsigned)r[1]);
    return (threadIdx.x & 32) ? a : b;
}

// ---------------------------------------------------------------------------------------------
// Tiles staged with direct global->LDS loads (global_load_lds_dwordx4).
// One such instruction makes a wave write 64 x 16 B = 1 KB of consecutive LDS, so rows cannot be
// padded; bank conflicts are avoided by permuting the 16-byte chunks of each row instead: chunk
// ch of tile row r is stored at chunk position ch ^ swz(r).  With swz even and periodic in 8 rows
// (of 256 B) the 8 lanes of a row-wise 16-byte read and the 4 rows of a transposing read each fall
// on distinct banks.  CH = chunks per row (D / 8).
template <int CH>
__device__ __forceinline__ int swz(int r) { return 2 * ((r * CH / 16) % (CH / 2)); }

// byte offset of (row r, chunk ch) inside a swizzled tile
template <int CH>
__device__ __forceinline__ int swz_off(int r, int ch) { return r * (CH * 16) + ((ch ^ swz<CH>(r)) << 4); }

// issue one 1 KB direct load: lane `lane` fetches 16 bytes from `src` into lds_base + 16 * lane
__device__ __forceinline__ void g2l16(const void* src, void* lds_base_uniform) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                     (__attribute__((address_space(3))) void*)lds_base_uniform, 16, 0, 0);
}

// wait until this wave's outstanding vector-memory operations (direct loads included) are done
__device__ __forceinline__ void wait_vmem() { __builtin_amdgcn_s_waitcnt(0x0F70); }

template <int CH>
__device__ __forceinline__ int tr_lane_row() {
    const int lane = threadIdx.x & 63;
    return 4 * (lane >> 5) + ((lane & 15) >> 2);
}
// A operand X^T from a swizzled row-major LDS tile X[row][col]: the lane gets, for column col0 + lane % 32,
// the 8 rows row0 + 4h + {0,1,2,3} and row0 + 8 + 4h + {0,1,2,3} (row0 a multiple of 8, col0 = 32 db) with two
// ds_read_b64_tr_b16: within each 16-lane group, lane p passes the address of X[r + p/4][c + 4 (p%4)] and
// receives X[r .. r+3][c + p].  The address is split into a per-lane register tr_lane_off<CH>(db),
// computed once per kernel, and compile-time parts (rows, LDS stage) that become immediates.
template <int CH>
__device__ __forceinline__ int tr_lane_off(int db) {
    const int lane = threadIdx.x & 63;
    const int p16 = lane & 15, gi2 = (lane >> 4) & 1;
    const int rl = tr_lane_row<CH>();
    const int ch = 4 * db + 2 * gi2 + ((p16 & 3) >> 1);
    return rl * (CH * 16) + ((ch ^ swz<CH>(rl)) << 4) + (p16 & 1) * 8;
}
template <int CH>
__device__ __forceinline__ bf16x8 tr16_frag_at(const char* tile_plus_lane_off, int row0) {
    const char* a = tile_plus_lane_off + row0 * (CH * 16);
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)a);
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(a + 8 * CH * 16));
    s16x8 r = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, r);
}

// 8 consecutive C registers (starting at i0) -> bf16 B operand
__device__ __forceinline__ bf16x8 pack8(const f32x16& x, int i0) {
    u32x4 r;
    r[0] = pack_bf16x2(x[i0], x[i0 + 1]);
    r[1] = pack_bf16x2(x[i0 + 2], x[i0 + 3]);
    r[2] = pack_bf16x2(x[i0 + 4], x[i0 + 5]);
    r[3] = pack_bf16x2(x[i0 + 6], x[i0 + 7]);
    return __builtin_bit_cast(bf16x8, r);
}


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
