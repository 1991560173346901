// Entry points that launch nothing: version, error names, workspace sizes.
#include "common.hpp"

namespace fastar {
size_t compress_ws_bytes(int H, int C, int n_new, int r);
size_t select_self_ws_bytes(int H, int n_q, int C, int r, int BQ, int BK, int n_rep);
size_t select_cross_ws_bytes(int H, int n_q, int n_p, int BQ);
size_t select_lsh_ws_bytes(int H, int n_q, int C, int n_bits, int BQ, int BK, int n_rep);
size_t select_buckets_ws_bytes(int H, int n_q, int C, int n_p, int BQ, int BK);
size_t attn_sk_ws_bytes();
}  // namespace fastar

namespace fastar {

// Register-resident matrix-core loop: four independent bf16 32x32x16 accumulators per wavefront, no memory traffic.
// RANDOM = false: every operand element is 1.0 / 0.5 (the data path hardly toggles); true: operands drawn per lane from
// a hash, uniform in (-2, 2), four different pairs per wavefront (what real keys and queries look like to the
// multipliers).  The chip's clock under the two differs, which is what the second one is for.
template <bool RANDOM>
__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters, float *sink) {
    bf16x8 a[4], b[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (RANDOM) {
                unsigned x = (threadIdx.x * 64u + j * 8u + i) + blockIdx.x * 7919u;
                x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
                a[j][i] = (__bf16)(((int)(x & 0xFFFF) - 32768) / 16384.0f);
                b[j][i] = (__bf16)(((int)(x >> 16) - 32768) / 16384.0f);
            } else {
                a[j][i] = (__bf16)1.0f;
                b[j][i] = (__bf16)0.5f;
            }
        }
    f32x16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.0f;
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] = mfma_bf16_32x32x16(a[j], b[j], acc[j]);
    }
    if (acc[0][0] + acc[1][1] + acc[2][2] + acc[3][3] == 12345.0f) sink[0] = 1.0f;
}

// Plain streaming copy, 16 bytes per lane, grid-stride.
__global__ __launch_bounds__(256) void probe_copy_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, size_t n16) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x)
        dst[i] = src[i];
}

}  // namespace fastar

extern "C" int fastar_probe_mfma_bf16(int iters, int random_operands, float *sink, double *flops_out, void *stream) {
    if (iters <= 0 || !sink) return FASTAR_ERR_INVALID_ARG;
    const int wgs = 256 * 8;
    if (random_operands)
        hipLaunchKernelGGL(fastar::probe_mfma_kernel<true>, dim3(wgs), dim3(256), 0, (hipStream_t)stream, iters, sink);
    else
        hipLaunchKernelGGL(fastar::probe_mfma_kernel<false>, dim3(wgs), dim3(256), 0, (hipStream_t)stream, iters, sink);
    if (hipGetLastError() != hipSuccess) return FASTAR_ERR_HIP;
    if (flops_out) *flops_out = (double)wgs * 4.0 * (double)iters * 4.0 * 32768.0;
    return FASTAR_OK;
}

extern "C" int fastar_probe_copy(const void *src, void *dst, size_t bytes, void *stream) {
    if (!src || !dst || (bytes & 15) || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15)) return FASTAR_ERR_INVALID_ARG;
    hipLaunchKernelGGL(fastar::probe_copy_kernel, dim3(256 * 16), dim3(256), 0, (hipStream_t)stream,
                       (const fastar::u32x4 *)src, (fastar::u32x4 *)dst, bytes / 16);
    if (hipGetLastError() != hipSuccess) return FASTAR_ERR_HIP;
    return FASTAR_OK;
}

extern "C" int fastar_init(void) {
    int rc = fastar::attn_d128_pp_setup();
    if (rc == FASTAR_OK) rc = fastar::attn_d128_setup();
    if (rc == FASTAR_OK) rc = fastar::select_setup();
    if (rc == FASTAR_OK) rc = fastar::tempcache_setup();
    if (rc == FASTAR_OK) rc = fastar::attn_fp8_setup();
    return rc;
}

extern "C" const char *fastar_version(void) { return "fastar-gfx950 0.1"; }

extern "C" const char *fastar_strerror(int code) {
    switch (code) {
        case FASTAR_OK: return "ok";
        case FASTAR_ERR_INVALID_ARG: return "invalid argument";
        case FASTAR_ERR_UNSUPPORTED: return "unsupported shape or type";
        case FASTAR_ERR_WORKSPACE: return "workspace too small";
        case FASTAR_ERR_HIP: return "HIP launch error";
        case FASTAR_ERR_STATIC_SCRATCH: return "problem larger than the library's static scratch";
        default: return "unknown error";
    }
}

extern "C" size_t fastar_workspace_bytes(int op, int H, int n_q, int n_k, int r, int BQ, int BK, int n_rep) {
    switch (op) {
        case FASTAR_OP_COMPRESS: return fastar::compress_ws_bytes(H, n_k, n_q, r);
        case FASTAR_OP_SELECT_SELF: return fastar::select_self_ws_bytes(H, n_q, n_k, r, BQ, BK, n_rep);
        case FASTAR_OP_SELECT_CROSS: return fastar::select_cross_ws_bytes(H, n_q, n_k, BQ);
        case FASTAR_OP_SELECT_LSH: return fastar::select_lsh_ws_bytes(H, n_q, n_k, r, BQ, BK, n_rep);
        case FASTAR_OP_SELECT_BUCKETS: return fastar::select_buckets_ws_bytes(H, n_q, n_k, r, BQ, BK);
        case FASTAR_OP_ATTN: return fastar::attn_sk_ws_bytes();
        default: return 0;
    }
}
