// Device pieces of the ANN code (Sec. 5.1 of the paper), shared by the encode kernels and by the TempCache
// match kernel that encodes its own probes:
//   xq = clamp(rint(x * qscale), +-127);  y = R^T xq (int32);  c = clamp((y + 2^(sh-1)) >> sh, +-127)
// One wavefront owns 16 vectors at a time: B operand = their quantised coordinates (column = vector), A operand =
// R^T (row = code coordinate), accumulator row 4*(lane/16)+v / column lane%16, so a lane ends up with 4
// consecutive code bytes of one vector.
#pragma once
#include "common.hpp"

namespace fastar {

// Coordinate t that k-slot e (0..15) of quarter g stands for in k-step ks.  Chosen so that each
// 16-byte load of a lane is contiguous and the four quarters of a row tile the row.
template <bool BF16>
__device__ __forceinline__ int slot_coord(int ks, int g, int e) {
    if (BF16) return ks * 64 + (e >> 3) * 32 + 8 * g + (e & 7);
    return ks * 64 + (e >> 2) * 16 + 4 * g + (e & 3);
}

// Quantised coordinates of one vector for k-step ks, as the 16 int8 k-slots of this lane.
template <bool BF16>
__device__ __forceinline__ i32x4 load_quantised(const void *row, int ks, int g, float qscale) {
    i32x4 out;
    if (BF16) {
        const unsigned short *p = (const unsigned short *)row;
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            u32x4 w = *(const u32x4 *)(p + ks * 64 + m * 32 + 8 * g);
            int q[8];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                q[2 * e] = quant8(bf16_lo(w[e]), qscale);
                q[2 * e + 1] = quant8(bf16_hi(w[e]), qscale);
            }
            out[2 * m] = (int)pack_i8x4(q[0], q[1], q[2], q[3]);
            out[2 * m + 1] = (int)pack_i8x4(q[4], q[5], q[6], q[7]);
        }
    } else {
        const float *p = (const float *)row;
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            f32x4 w = *(const f32x4 *)(p + ks * 64 + m * 16 + 4 * g);
            out[m] = (int)pack_i8x4(quant8(w[0], qscale), quant8(w[1], qscale), quant8(w[2], qscale), quant8(w[3], qscale));
        }
    }
    return out;
}

__device__ __forceinline__ int requant(int y, int shift) {
    int c = (y + (1 << (shift - 1))) >> shift;  // arithmetic shift = floor division
    return min(max(c, -127), 127);
}

// A operand of one wavefront: rows of R^T for every (k-step of 64 coordinates, block of 16 code coordinates).
template <bool BF16, int D, int R>
struct CodeMatrix {
    static constexpr int KS = D / 64, CB = R / 16;
    i32x4 a[KS][CB];
    __device__ __forceinline__ void load(const int8_t *__restrict__ Rm, int lane) {
        const int col = lane & 15, g = lane >> 4;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
                int b[16];
#pragma unroll
                for (int e = 0; e < 16; ++e) b[e] = Rm[slot_coord<BF16>(ks, g, e) * R + cb * 16 + col];
#pragma unroll
                for (int m = 0; m < 4; ++m) a[ks][cb][m] = (int)pack_i8x4(b[4 * m], b[4 * m + 1], b[4 * m + 2], b[4 * m + 3]);
            }
    }
    // Code bytes cb*16 + 4*(lane/16) .. +3 of the vector whose quantised coordinates are b (column lane%16).
    __device__ __forceinline__ unsigned code_word(const i32x4 (&b)[KS], int cb, int shift) const {
        i32x4 acc = {0, 0, 0, 0};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) acc = mfma_i8_16x16x64(a[ks][cb], b[ks], acc);
        return pack_i8x4(requant(acc[0], shift), requant(acc[1], shift), requant(acc[2], shift), requant(acc[3], shift));
    }
    // The same four entries at BITS (2 or 4) bits each, saturated to +-(2^(BITS-1) - 1), entry v in bits [BITS*v, +BITS).
    template <int BITS>
    __device__ __forceinline__ unsigned code_bits(const i32x4 (&b)[KS], int cb, int shift) const {
        i32x4 acc = {0, 0, 0, 0};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) acc = mfma_i8_16x16x64(a[ks][cb], b[ks], acc);
        constexpr int LIM = (1 << (BITS - 1)) - 1;
        unsigned w = 0;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int c = min(max((acc[v] + (1 << (shift - 1))) >> shift, -LIM), LIM);
            w |= ((unsigned)c & ((1u << BITS) - 1u)) << (BITS * v);
        }
        return w;
    }
};

}  // namespace fastar
