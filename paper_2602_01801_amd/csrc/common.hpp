// Shared device helpers of libfastar (gfx950 only): vector types, MFMA wrappers, bf16 handling,
// the 8-bit quantiser and wave-level primitives.  Wavefronts are 64 lanes wide throughout.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <mutex>

#include "../../include/fastar.h"

namespace fastar {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) int i32x2;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(16))) int i32x16;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

constexpr int WAVE = 64;

// ---- MFMA ---------------------------------------------------------------------------------------
// 32x32 tiles: lane l supplies row (A) / column (B) l%32 and the k-slots of half g = l/32; the
// accumulator register v of lane l is element (row 8*(v/4) + 4*g + v%4, column l%32).
// 16x16 tiles: lane l supplies row / column l%16 and the k-slots of quarter l/16; accumulator
// register v is element (row 4*(l/16) + v, column l%16).
// Which k a slot stands for is free as long as A and B agree, so operands are loaded with whatever
// k order suits the memory layout.

__device__ __forceinline__ f32x16 mfma_bf16_32x32x16(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ i32x16 mfma_i8_32x32x32(i32x4 a, i32x4 b, i32x16 c) {
    return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ i32x4 mfma_i8_16x16x64(i32x4 a, i32x4 b, i32x4 c) {
    return __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, c, 0, 0, 0);
}

// ---- bf16 ---------------------------------------------------------------------------------------

__device__ __forceinline__ float bf16_bits_to_f32(unsigned short b) { return __uint_as_float(((unsigned)b) << 16); }
__device__ __forceinline__ float bf16_lo(unsigned w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(unsigned w) { return __uint_as_float(w & 0xFFFF0000u); }

// float -> bfloat16 bits, nearest with ties to even (inputs are finite here).
__device__ __forceinline__ unsigned f32_to_bf16_bits(float f) {
    unsigned u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}
__device__ __forceinline__ unsigned pack_bf16x2(float lo, float hi) {
    return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

// ---- quantiser of the ANN code ----------------------------------------------------------------------
// One float32 multiply, round half to even, saturate to [-127, 127].
__device__ __forceinline__ int quant8(float x, float qscale) {
    float p = __fmul_rn(x, qscale);
    float q = rintf(p);
    q = fminf(fmaxf(q, -127.0f), 127.0f);
    return (int)q;
}
__device__ __forceinline__ unsigned pack_i8x4(int a, int b, int c, int d) {
    return (unsigned)(a & 0xFF) | ((unsigned)(b & 0xFF) << 8) | ((unsigned)(c & 0xFF) << 16) | ((unsigned)(d & 0xFF) << 24);
}

// ---- wave primitives ------------------------------------------------------------------------------

__device__ __forceinline__ int lane_id() { return threadIdx.x & (WAVE - 1); }

template <typename T>
__device__ __forceinline__ T shfl_xor(T v, int mask) {
    return __shfl_xor(v, mask, WAVE);
}

__device__ __forceinline__ int dot4_i8(unsigned a, unsigned b, int acc) {
    return __builtin_amdgcn_sdot4((int)a, (int)b, acc, false);
}

// One-time set-up per device (kernel attributes, symbol addresses), safe to reach from several host threads: run(f)
// calls f once per device ordinal, with that device current, and remembers a success.  It is the only process-wide data
// the library keeps, and it never influences a result.
struct DeviceOnce {
    static constexpr int MAX_DEVICES = 64;
    std::atomic<unsigned long long> done{0};
    std::mutex mu;
    template <class F>
    int run(F &&f) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess) return FASTAR_ERR_HIP;
        if (dev < 0 || dev >= MAX_DEVICES) return FASTAR_ERR_UNSUPPORTED;
        const unsigned long long bit = 1ull << dev;
        if (done.load(std::memory_order_acquire) & bit) return FASTAR_OK;
        std::lock_guard<std::mutex> lock(mu);
        if (done.load(std::memory_order_relaxed) & bit) return FASTAR_OK;
        const int rc = f(dev);
        if (rc == FASTAR_OK) done.fetch_or(bit, std::memory_order_release);
        return rc;
    }
};

// ---- split attention launches (sparse_attn_fwd_ws, sparse_attn_fwd_fp8_ws) ---------------------------------------
// The (head, query block) pairs are dealt to the 8 XCDs in contiguous ranges of `per`; the first `full_per` pairs of every
// range are taken by one workgroup each, the others are cut into equal shares of their tiles (attention_d128.hip).
struct TailMap {
    int per, full_per, total;   // pairs per XCD range, of them taken whole, pairs in all
    __host__ __device__ __forceinline__ int tail_per() const { return per - full_per; }
    __host__ __device__ __forceinline__ long long tiles(int NT) const { return (long long)8 * tail_per() * NT; }
    // position in the left-over sequence -> (head, block) pair; pairs >= total do not exist (the last range may be short)
    __host__ __device__ __forceinline__ int item(int vi) const { return (vi / tail_per()) * per + full_per + vi % tail_per(); }
};
constexpr int ATTN_SHARE_WORKGROUPS = 512;                      // resident workgroups that take the shares: two per CU
constexpr int ATTN_PART_O_FLOATS = (128 / 32) * 16 * 64;        // O^T accumulators of one wavefront (d = 128)
constexpr int ATTN_PART_FLOATS = 4 * (ATTN_PART_O_FLOATS + 2 * 64);   // one fragment of a query block: four wavefronts' accumulators, reference maxima, row sums
// Whether a launch of n_items pairs with n_tiles 64-key tiles each is split, and how many pairs per range are taken
// whole then (0: not split).  What the split saves: a last round of n_tiles tiles at a lone workgroup's pace (about 1.2 us
// per tile) against tail_per / 64 of a round at the pace of a full chip (2.4 us per tile) plus about 30 us of fragments and
// launches (an XCD holds 64 workgroups of the one-block kernels).
inline int attn_split_full_per(int n_items, int n_tiles) {
    const int per_xcd = (n_items + 7) / 8, tail_per = per_xcd % 64;
    if (per_xcd > 64 && tail_per > 0 && tail_per <= 24 && (float)n_tiles * (1.2f - 0.0375f * (float)tail_per) > 30.0f)
        return per_xcd - tail_per;
    return 0;
}
int launch_attn_combine(const void *ws, int n_q, int n_qb, TailMap tm, int NT, float scale_log2, float lse_offset, void *O,
                        float *lse, hipStream_t s);

// Per-file set-up, all of it run by fastar_init() (api.hip) and each lazily by the first launch that needs it.
int attn_d128_pp_setup();
int attn_d128_setup();
int select_setup();
int tempcache_setup();
int attn_fp8_setup();

// Host-side launch check shared by the entry points.
#define FASTAR_LAUNCH_CHECK()                          \
    do {                                               \
        if (hipGetLastError() != hipSuccess) return FASTAR_ERR_HIP; \
    } while (0)

}  // namespace fastar
