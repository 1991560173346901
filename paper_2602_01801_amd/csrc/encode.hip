// ANN codes (Sec. 5.1 of the paper: shared low-dimensional random projection + 8-bit quantisation).
//
//   xq = clamp(rint(x * qscale), +-127);  y = R^T xq (int32);  c = clamp((y + 2^(sh-1)) >> sh, +-127)
//
// HBM-bound: d*es bytes in, r bytes out per vector; the d x r contraction (2*d*r integer ops per
// vector) runs on the int8 matrix cores so that it stays off the critical path.  One wavefront owns
// 16 vectors at a time: B operand = their quantised coordinates (column = vector), A operand = R^T
// (row = code coordinate), accumulator row 4*(lane/16)+v / column lane%16, so a lane ends up with 4
// consecutive code bytes of one vector and stores them as one dword.
#include "encode_dev.hpp"

namespace fastar {

template <bool BF16, int D, int R>
__global__ __launch_bounds__(256) void encode_kernel(const void *__restrict__ x, int64_t n_vec,
                                                     const int8_t *__restrict__ Rm, float qscale, int shift,
                                                     int8_t *__restrict__ code, unsigned long long *zero_fill,
                                                     int64_t zero_n) {
    constexpr int KS = D / 64;   // k-steps of 64 coordinates
    constexpr int CB = R / 16;   // blocks of 16 code coordinates
    const int lane = lane_id();
    const int col = lane & 15, g = lane >> 4;
    const int64_t gtid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t gthreads = (int64_t)gridDim.x * blockDim.x;
    // optional: clear a 64-bit array for a later kernel of the same call
    for (int64_t i = gtid; i < zero_n; i += gthreads) zero_fill[i] = 0ull;

    // A operand: rows of R^T for every (k-step, code block), gathered once per wavefront
    CodeMatrix<BF16, D, R> cm;
    cm.load(Rm, lane);

    const int64_t wave = gtid >> 6, n_waves = gthreads >> 6;
    const int64_t n_groups = (n_vec + 15) >> 4;
    const size_t row_bytes = (size_t)D * (BF16 ? 2 : 4);
    for (int64_t grp = wave; grp < n_groups; grp += n_waves) {
        const int64_t vec = grp * 16 + col;
        const int64_t vload = vec < n_vec ? vec : n_vec - 1;
        const char *row = (const char *)x + (size_t)vload * row_bytes;
        i32x4 b[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) b[ks] = load_quantised<BF16>(row, ks, g, qscale);
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            const unsigned w = cm.code_word(b, cb, shift);
            if (vec < n_vec) *(unsigned *)(code + vec * R + cb * 16 + 4 * g) = w;
        }
    }
}

template <bool BF16, int D, int R>
static void launch_encode(const void *x, int64_t n_vec, const fastar_codec *codec, int8_t *code,
                          unsigned long long *zero_fill, int64_t zero_n, hipStream_t s) {
    int64_t groups = (n_vec + 15) / 16;
    int64_t blocks = (groups + 3) / 4;
    if (blocks > 4096) blocks = 4096;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL((encode_kernel<BF16, D, R>), dim3((unsigned)blocks), dim3(256), 0, s, x, n_vec, codec->R,
                       codec->qscale, codec->shift, code, zero_fill, zero_n);
}

// Internal launcher shared with tempcache_compress: encodes and optionally zero-fills an array.
int encode_launch(const void *x, int dtype, int64_t n_vec, int d, const fastar_codec *codec, int r, int8_t *code,
                  unsigned long long *zero_fill, int64_t zero_n, hipStream_t s) {
    if (!x || !codec || !codec->R || !code || n_vec < 0) return FASTAR_ERR_INVALID_ARG;
    if (dtype != FASTAR_F32 && dtype != FASTAR_BF16) return FASTAR_ERR_INVALID_ARG;
    if (codec->shift < 1 || codec->shift > 16) return FASTAR_ERR_INVALID_ARG;
    if ((d != 64 && d != 128) || (r != 32 && r != 64)) return FASTAR_ERR_UNSUPPORTED;
    if (((uintptr_t)x & 15) || ((uintptr_t)code & 3)) return FASTAR_ERR_INVALID_ARG;
    if (n_vec == 0 && zero_n == 0) return FASTAR_OK;
#define FASTAR_ENC(B, DD, RR) launch_encode<B, DD, RR>(x, n_vec, codec, code, zero_fill, zero_n, s)
    const bool bf = dtype == FASTAR_BF16;
    if (d == 64 && r == 32) { if (bf) FASTAR_ENC(true, 64, 32); else FASTAR_ENC(false, 64, 32); }
    else if (d == 64 && r == 64) { if (bf) FASTAR_ENC(true, 64, 64); else FASTAR_ENC(false, 64, 64); }
    else if (d == 128 && r == 32) { if (bf) FASTAR_ENC(true, 128, 32); else FASTAR_ENC(false, 128, 32); }
    else { if (bf) FASTAR_ENC(true, 128, 64); else FASTAR_ENC(false, 128, 64); }
#undef FASTAR_ENC
    FASTAR_LAUNCH_CHECK();
    return FASTAR_OK;
}

// ---- codes of 2 or 4 bits per entry, packed (appendix, "Quantization precision for ANN matching") -------------------
// Same operands as encode_kernel; a lane ends with four entries of one vector = BITS / 2 bytes.
template <bool BF16, int D, int R, int BITS>
__global__ __launch_bounds__(256) void encode_packed_kernel(const void *__restrict__ x, int64_t n_vec,
                                                            const int8_t *__restrict__ Rm, float qscale, int shift,
                                                            uint8_t *__restrict__ packed) {
    constexpr int KS = D / 64, CB = R / 16;
    constexpr int ROWB = R * BITS / 8;
    const int lane = lane_id();
    const int col = lane & 15, g = lane >> 4;
    CodeMatrix<BF16, D, R> cm;
    cm.load(Rm, lane);
    const int64_t gtid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t wave = gtid >> 6, n_waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    const int64_t n_groups = (n_vec + 15) >> 4;
    const size_t row_bytes = (size_t)D * (BF16 ? 2 : 4);
    for (int64_t grp = wave; grp < n_groups; grp += n_waves) {
        const int64_t vec = grp * 16 + col;
        const int64_t vload = vec < n_vec ? vec : n_vec - 1;
        const char *row = (const char *)x + (size_t)vload * row_bytes;
        i32x4 b[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) b[ks] = load_quantised<BF16>(row, ks, g, qscale);
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            const unsigned w = cm.template code_bits<BITS>(b, cb, shift);
            if (vec < n_vec) {
                uint8_t *dst = packed + vec * ROWB + (cb * 16 + 4 * g) * BITS / 8;
                if (BITS == 4) *(unsigned short *)dst = (unsigned short)w;
                else *dst = (uint8_t)w;
            }
        }
    }
}

// ---- sign codes (LSH paragraph of Sec. 5.1): bit j = [ (R^T xq)_j >= 0 ] --------------------------------------
// Same operand layout as encode_kernel; NB hash bits = NB/16 blocks of 16 rows of R^T.  A lane ends with the 4 sign
// bits (rows 4g+v of a block) of one vector per block; two blocks and the four quarters g make one 32-bit word,
// combined across the quarters with two lane exchanges.
template <bool BF16, int D, int NB>
__global__ __launch_bounds__(256) void encode_sign_kernel(const void *__restrict__ x, int64_t n_vec,
                                                          const int8_t *__restrict__ Rm, float qscale,
                                                          uint32_t *__restrict__ bits) {
    constexpr int KS = D / 64;
    constexpr int CB = NB / 16;
    constexpr int W = NB / 32;
    const int lane = lane_id();
    const int col = lane & 15, g = lane >> 4;
    const int64_t gtid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t gthreads = (int64_t)gridDim.x * blockDim.x;
    i32x4 a[KS][CB];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            int b[16];
#pragma unroll
            for (int e = 0; e < 16; ++e) b[e] = Rm[slot_coord<BF16>(ks, g, e) * NB + cb * 16 + col];
#pragma unroll
            for (int m = 0; m < 4; ++m) a[ks][cb][m] = (int)pack_i8x4(b[4 * m], b[4 * m + 1], b[4 * m + 2], b[4 * m + 3]);
        }
    const int64_t wave = gtid >> 6, n_waves = gthreads >> 6;
    const int64_t n_groups = (n_vec + 15) >> 4;
    const size_t row_bytes = (size_t)D * (BF16 ? 2 : 4);
    for (int64_t grp = wave; grp < n_groups; grp += n_waves) {
        const int64_t vec = grp * 16 + col;
        const int64_t vload = vec < n_vec ? vec : n_vec - 1;
        const char *row = (const char *)x + (size_t)vload * row_bytes;
        i32x4 b[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) b[ks] = load_quantised<BF16>(row, ks, g, qscale);
#pragma unroll
        for (int w = 0; w < W; ++w) {
            unsigned word = 0;
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const int cb = 2 * w + half;
                i32x4 acc = {0, 0, 0, 0};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) acc = mfma_i8_16x16x64(a[ks][cb], b[ks], acc);
                unsigned nib = 0;
#pragma unroll
                for (int v = 0; v < 4; ++v) nib |= (acc[v] >= 0 ? 1u : 0u) << v;
                word |= nib << (16 * half + 4 * g);
            }
            word |= shfl_xor(word, 16);
            word |= shfl_xor(word, 32);
            if (g == 0 && vec < n_vec) bits[vec * W + w] = word;
        }
    }
}

template <bool BF16, int D, int NB>
static void launch_encode_sign(const void *x, int64_t n_vec, const int8_t *R, float qscale, uint32_t *bits,
                               hipStream_t s) {
    int64_t groups = (n_vec + 15) / 16;
    int64_t blocks = (groups + 3) / 4;
    if (blocks > 4096) blocks = 4096;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL((encode_sign_kernel<BF16, D, NB>), dim3((unsigned)blocks), dim3(256), 0, s, x, n_vec, R, qscale,
                       bits);
}

}  // namespace fastar

extern "C" int fastar_encode(const void *x, int dtype, int64_t n_vec, int d, const fastar_codec *codec, int r,
                             int8_t *code_out, void *stream) {
    return fastar::encode_launch(x, dtype, n_vec, d, codec, r, code_out, nullptr, 0, (hipStream_t)stream);
}

extern "C" int fastar_encode_packed(const void *x, int dtype, int64_t n_vec, int d, const fastar_codec *codec, int r,
                                    int bits, uint8_t *packed_out, void *stream) {
    using namespace fastar;
    if (bits == 8) return encode_launch(x, dtype, n_vec, d, codec, r, (int8_t *)packed_out, nullptr, 0, (hipStream_t)stream);
    if (!x || !codec || !codec->R || !packed_out || n_vec < 0) return FASTAR_ERR_INVALID_ARG;
    if (dtype != FASTAR_F32 && dtype != FASTAR_BF16) return FASTAR_ERR_INVALID_ARG;
    if (bits != 2 && bits != 4) return FASTAR_ERR_INVALID_ARG;
    if (codec->shift < 1 || codec->shift > 16) return FASTAR_ERR_INVALID_ARG;
    if ((d != 64 && d != 128) || r != 32) return FASTAR_ERR_UNSUPPORTED;
    if (((uintptr_t)x & 15) || ((uintptr_t)packed_out & 3)) return FASTAR_ERR_INVALID_ARG;
    if (n_vec == 0) return FASTAR_OK;
    hipStream_t s = (hipStream_t)stream;
    int64_t blocks = ((n_vec + 15) / 16 + 3) / 4;
    if (blocks > 4096) blocks = 4096;
#define FASTAR_ENCP(B, DD, BB)                                                                                       \
    hipLaunchKernelGGL((encode_packed_kernel<B, DD, 32, BB>), dim3((unsigned)blocks), dim3(256), 0, s, x, n_vec, codec->R, \
                       codec->qscale, codec->shift, packed_out)
    const bool bf = dtype == FASTAR_BF16;
    if (d == 64) {
        if (bits == 4) { if (bf) FASTAR_ENCP(true, 64, 4); else FASTAR_ENCP(false, 64, 4); }
        else { if (bf) FASTAR_ENCP(true, 64, 2); else FASTAR_ENCP(false, 64, 2); }
    } else {
        if (bits == 4) { if (bf) FASTAR_ENCP(true, 128, 4); else FASTAR_ENCP(false, 128, 4); }
        else { if (bf) FASTAR_ENCP(true, 128, 2); else FASTAR_ENCP(false, 128, 2); }
    }
#undef FASTAR_ENCP
    FASTAR_LAUNCH_CHECK();
    return FASTAR_OK;
}

extern "C" int fastar_encode_sign(const void *x, int dtype, int64_t n_vec, int d, const int8_t *R, float qscale,
                                  int n_bits, uint32_t *bits_out, void *stream) {
    using namespace fastar;
    if (!x || !R || !bits_out || n_vec < 0) return FASTAR_ERR_INVALID_ARG;
    if (dtype != FASTAR_F32 && dtype != FASTAR_BF16) return FASTAR_ERR_INVALID_ARG;
    if ((d != 64 && d != 128) || (n_bits != 64 && n_bits != 128 && n_bits != 256)) return FASTAR_ERR_UNSUPPORTED;
    if (((uintptr_t)x & 15) || ((uintptr_t)bits_out & 3)) return FASTAR_ERR_INVALID_ARG;
    if (n_vec == 0) return FASTAR_OK;
    hipStream_t s = (hipStream_t)stream;
    const bool bf = dtype == FASTAR_BF16;
#define FASTAR_ENCS(DD, NB)                                                              \
    do {                                                                                 \
        if (bf) launch_encode_sign<true, DD, NB>(x, n_vec, R, qscale, bits_out, s);      \
        else launch_encode_sign<false, DD, NB>(x, n_vec, R, qscale, bits_out, s);        \
    } while (0)
    if (d == 64 && n_bits == 64) FASTAR_ENCS(64, 64);
    else if (d == 64 && n_bits == 128) FASTAR_ENCS(64, 128);
    else if (d == 64) FASTAR_ENCS(64, 256);
    else if (n_bits == 64) FASTAR_ENCS(128, 64);
    else if (n_bits == 128) FASTAR_ENCS(128, 128);
    else FASTAR_ENCS(128, 256);
#undef FASTAR_ENCS
    FASTAR_LAUNCH_CHECK();
    return FASTAR_OK;
}
