// Prompt-induced buckets for self-attention (Sec. 5.4, first paragraph: AnnSA reuses the semantic buckets that
// cross-attention pruning found; a query belongs to one or more buckets and attends only to keys of the same bucket(s)).
//
// The prompt tokens are the buckets.  Four small kernels, all on exact integers:
//   prompt_bucket_kernel   the m nearest prompt tokens of every code (the products AnnCA ranks prompt tokens by, on
//                          the int8 matrix cores; one packed 32-bit key per product keeps "largest product, then
//                          smallest token" under a plain unsigned maximum)
//   bucket_mask_kernel     one bit per prompt token: the buckets a query block / key block owns, stored word-major so
//                          that the scoring reads them coalesced
//   bucket_score_kernel    shared buckets of every (query block, key block) pair: AND + bit count
//   bucket_topk_kernel     candidates (at least one shared bucket, or forced) counted, then the exact top-k of select.hip
#include <algorithm>

#include "common.hpp"
#include "topk_dev.hpp"

namespace fastar {

constexpr int BUCKET_MAX_PROMPT = 2048;   // 11 bits of a packed key hold the token id
constexpr int MASK_BLOCKS_PER_WG = 64;

// ---- nearest prompt tokens ---------------------------------------------------------------------------------------
// D = A x B with A rows = 32 prompt tokens, B columns = 32 codes: a lane ends with 16 products of ONE code (column
// lane % 32) with prompt tokens pb*32 + 8(v/4) + 4(lane/32) + v%4, ascending in v.
// key = (product + 2^20) * 2^11 + (2047 - token): |product| <= 64 * 127^2 < 2^20, token < 2^11.
// Bucket j of a code is the largest key below bucket j-1's: pass j repeats the products (they are cheap) with that bound.
template <int R>
__global__ __launch_bounds__(256) void prompt_bucket_kernel(const int8_t *__restrict__ code, int C,
                                                            const int32_t *__restrict__ idx, int n,
                                                            const int8_t *__restrict__ pcode, int n_p, int m,
                                                            int32_t *__restrict__ bucket) {
    constexpr int KS = R / 32;
    const int h = blockIdx.y;
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int col = lane & 31, g = lane >> 5;
    const int li = blockIdx.x * 128 + wave * 32 + col;
    int slot = -1;
    if (li < n) slot = idx ? idx[(size_t)h * n + li] : li;
    if (slot >= C) slot = -1;
    const int8_t *crow = code + ((size_t)h * C + max(slot, 0)) * R;
    i32x4 bfrag[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) bfrag[ks] = *(const i32x4 *)(crow + ks * 32 + 16 * g);
    unsigned cv[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) cv[v] = 0x80000000u + 2047u - (unsigned)(8 * (v / 4) + 4 * g + v % 4);
    const int8_t *ph = pcode + (size_t)h * n_p * R;
    const int n_pb = (n_p + 31) / 32;

    unsigned prev = 0xFFFFFFFFu;
    for (int j = 0; j < m; ++j) {
        unsigned best = 0;
        for (int pb = 0; pb < n_pb; pb += 4) {
            // four blocks of prompt tokens per step: their rows are loaded together, then multiplied
            i32x4 afrag[4][KS];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int prow = min((pb + u) * 32 + col, n_p - 1);   // rows past the end: any row, masked below
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) afrag[u][ks] = *(const i32x4 *)(ph + (size_t)prow * R + ks * 32 + 16 * g);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (pb + u < n_pb) {   // wave-uniform
                    i32x16 acc;
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[v] = 0;
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) acc = mfma_i8_32x32x32(afrag[u][ks], bfrag[ks], acc);
                    const unsigned shift = 32u * (unsigned)(pb + u);
                    // keys relative to this block (token id not yet lowered by 32 * block): compare against the
                    // bound raised by the same amount
                    const unsigned bound = j == 0 ? 0xFFFFFFFFu : prev + shift;
                    const int rows_left = n_p - 32 * (pb + u);   // < 32 in a ragged last block only
                    unsigned blk = 0;
                    if (rows_left >= 32) {
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const unsigned kr = ((unsigned)acc[v] << 11) + cv[v];
                            blk = max(blk, kr < bound ? kr : 0u);
                        }
                    } else {
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const unsigned kr = ((unsigned)acc[v] << 11) + cv[v];
                            const bool real = 8 * (v / 4) + 4 * g + v % 4 < rows_left;
                            blk = max(blk, (real && kr < bound) ? kr : 0u);
                        }
                    }
                    if (blk > 0) best = max(best, blk - shift);
                }
            }
        }
        best = max(best, (unsigned)__shfl_xor((int)best, 32, WAVE));
        if (g == 0 && slot >= 0) bucket[((size_t)h * C + slot) * m + j] = best ? 2047 - (int)(best & 2047u) : -1;
        prev = best;   // 0 once the prompt tokens are used up: nothing lies below it
    }
}

// ---- bucket masks of blocks ----------------------------------------------------------------------------------------
// mask[h][w][blk] bit t%32 of word w = t/32: some live row of block blk (BS consecutive rows of `bucket`) owns prompt
// token t.  A workgroup builds 64 blocks in LDS (one wavefront per block at a time) and writes them word-major.
__global__ __launch_bounds__(256) void bucket_mask_kernel(const int32_t *__restrict__ bucket, int N, int m,
                                                          const int32_t *__restrict__ len, int BS, int n_p, int W,
                                                          int n_blocks_cap, unsigned *__restrict__ mask) {
    extern __shared__ unsigned words[];   // [64][W + 1]
    const int h = blockIdx.y;
    const int blk0 = blockIdx.x * MASK_BLOCKS_PER_WG;
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int L = len ? min(len[h], N) : N;
    const int WP = W + 1;
    for (int t = threadIdx.x; t < MASK_BLOCKS_PER_WG * WP; t += 256) words[t] = 0;
    __syncthreads();
    for (int e = wave; e < MASK_BLOCKS_PER_WG; e += 4) {
        const int blk = blk0 + e;
        const long long row0 = (long long)blk * BS;
        const int rows = (int)max(0ll, min((long long)BS, (long long)L - row0));
        const int32_t *src = bucket + ((size_t)h * N + (size_t)max(row0, 0ll)) * m;
        for (int t = lane; t < rows * m; t += WAVE) {
            const int tok = src[t];
            if (tok >= 0 && tok < n_p) atomicOr(&words[e * WP + (tok >> 5)], 1u << (tok & 31));
        }
    }
    __syncthreads();
    for (int t = threadIdx.x; t < MASK_BLOCKS_PER_WG * W; t += 256) {
        const int w = t / MASK_BLOCKS_PER_WG, e = t % MASK_BLOCKS_PER_WG;
        if (blk0 + e < n_blocks_cap) mask[((size_t)h * W + w) * n_blocks_cap + blk0 + e] = words[e * WP + w];
    }
}

// ---- shared buckets of (query block, key block) pairs ---------------------------------------------------------------
// score[h][b][kb] = number of prompt tokens owned by both.  A thread owns a key block, eight query blocks at a time.
__global__ __launch_bounds__(256) void bucket_score_kernel(const unsigned *__restrict__ qmask, const unsigned *__restrict__ kmask,
                                                           int W, int n_qb, int n_kb_cap, int32_t *__restrict__ score) {
    extern __shared__ unsigned own[];   // [n_qb rounded up to 8][W], zero padded
    const int h = blockIdx.y;
    const int n_qb8 = (n_qb + 7) & ~7;
    for (int t = threadIdx.x; t < n_qb8 * W; t += 256) {
        const int b = t / W, w = t % W;
        own[t] = b < n_qb ? qmask[((size_t)h * W + w) * n_qb + b] : 0u;
    }
    __syncthreads();
    const int kb = blockIdx.x * 256 + threadIdx.x;
    if (kb >= n_kb_cap) return;
    const unsigned *km = kmask + (size_t)h * W * n_kb_cap + kb;
    for (int b0 = 0; b0 < n_qb; b0 += 8) {
        int acc[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = 0;
        for (int w = 0; w < W; ++w) {
            const unsigned mw = km[(size_t)w * n_kb_cap];
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] += __popc(mw & own[(b0 + e) * W + w]);
        }
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (b0 + e < n_qb) score[((size_t)h * n_qb + b0 + e) * n_kb_cap + kb] = acc[e];
    }
}

// ---- candidates, then the exact top-k -------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void bucket_topk_kernel(const int32_t *__restrict__ score, int n_kb_cap,
                                                          const int32_t *__restrict__ len, int C, int BK, int n_qb,
                                                          int n_sel, int n_sink, int n_local, int32_t *__restrict__ sel,
                                                          int32_t *__restrict__ nsel) {
    extern __shared__ unsigned keys[];   // min(n_kb_cap, TOPK_LDS_CAP) words: staging of the row's keys
    const int b = blockIdx.x, h = blockIdx.y;
    const int n = min((min(len[h], C) + BK - 1) / BK, n_kb_cap);
    const int32_t *row = score + ((size_t)h * n_qb + b) * n_kb_cap;
    const int n_cand = count_candidates(row, n, n_sink, n_local, 1);
    topk_row(row, n, n_sel, sel + ((size_t)h * n_qb + b) * n_sel, nsel + (size_t)h * n_qb + b, keys, n_sink, n_local,
             n_cand);
}

struct BucketWs {
    size_t qmask_off, kmask_off, score_off, total;
};
static inline size_t al256(size_t x) { return (x + 255) & ~(size_t)255; }
static BucketWs bucket_ws(int H, int n_q, int C, int n_p, int BQ, int BK) {
    const size_t W = (size_t)(n_p + 31) / 32;
    const size_t n_qb = (size_t)(n_q + BQ - 1) / BQ, n_kb = (size_t)(C + BK - 1) / BK;
    BucketWs w;
    w.qmask_off = 0;
    w.kmask_off = al256((size_t)H * W * n_qb * 4);
    w.score_off = w.kmask_off + al256((size_t)H * W * n_kb * 4);
    w.total = w.score_off + al256((size_t)H * n_qb * n_kb * 4);
    return w;
}
size_t select_buckets_ws_bytes(int H, int n_q, int C, int n_p, int BQ, int BK) {
    if (H <= 0 || n_q <= 0 || C <= 0 || n_p <= 0 || BQ <= 0 || BK <= 0) return 0;
    return bucket_ws(H, n_q, C, n_p, BQ, BK).total;
}

}  // namespace fastar

using namespace fastar;

extern "C" int ann_prompt_buckets(const int8_t *code, int C, const int32_t *idx, int n, const int8_t *pcode, int n_p,
                                  int H, int r, int m, int32_t *bucket, void *stream) {
    if (!code || !pcode || !bucket) return FASTAR_ERR_INVALID_ARG;
    if (H <= 0 || C <= 0 || n < 0 || n_p <= 0 || m <= 0) return FASTAR_ERR_INVALID_ARG;
    if (!idx && n > C) return FASTAR_ERR_INVALID_ARG;
    if (((uintptr_t)code & 15) || ((uintptr_t)pcode & 15)) return FASTAR_ERR_INVALID_ARG;
    if ((r != 32 && r != 64) || n_p > BUCKET_MAX_PROMPT || m > 8) return FASTAR_ERR_UNSUPPORTED;
    if (n == 0) return FASTAR_OK;
    const dim3 grid((unsigned)((n + 127) / 128), (unsigned)H);
    if (r == 32)
        hipLaunchKernelGGL(prompt_bucket_kernel<32>, grid, dim3(256), 0, (hipStream_t)stream, code, C, idx, n, pcode,
                           n_p, m, bucket);
    else
        hipLaunchKernelGGL(prompt_bucket_kernel<64>, grid, dim3(256), 0, (hipStream_t)stream, code, C, idx, n, pcode,
                           n_p, m, bucket);
    FASTAR_LAUNCH_CHECK();
    return FASTAR_OK;
}

extern "C" int ann_select_buckets(const int32_t *qbucket, int n_q, const int32_t *kbucket, const int32_t *len, int H,
                                  int C, int m, int n_p, int BQ, int BK, int n_sel, int n_sink, int n_local,
                                  int32_t *sel, int32_t *nsel, void *ws, size_t ws_bytes, void *stream) {
    if (!qbucket || !kbucket || !len || !sel || !nsel || !ws) return FASTAR_ERR_INVALID_ARG;
    if (H <= 0 || n_q <= 0 || C <= 0 || m <= 0 || n_p <= 0 || BQ <= 0 || BK <= 0 || n_sel <= 0)
        return FASTAR_ERR_INVALID_ARG;
    if (n_sink < 0 || n_local < 0 || n_sink + n_local > n_sel || ((uintptr_t)ws & 255)) return FASTAR_ERR_INVALID_ARG;
    if (n_p > BUCKET_MAX_PROMPT) return FASTAR_ERR_UNSUPPORTED;
    const int W = (n_p + 31) / 32;
    const int n_qb = (n_q + BQ - 1) / BQ, n_kb_cap = (C + BK - 1) / BK;
    const size_t own_bytes = (size_t)((n_qb + 7) & ~7) * W * 4;
    if (own_bytes > 48 * 1024) return FASTAR_ERR_UNSUPPORTED;   // the query blocks' masks of a head are staged in LDS
    const BucketWs w = bucket_ws(H, n_q, C, n_p, BQ, BK);
    if (ws_bytes < w.total) return FASTAR_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    unsigned *qmask = (unsigned *)((char *)ws + w.qmask_off);
    unsigned *kmask = (unsigned *)((char *)ws + w.kmask_off);
    int32_t *score = (int32_t *)((char *)ws + w.score_off);
    const size_t mask_lds = (size_t)MASK_BLOCKS_PER_WG * (W + 1) * 4;
    hipLaunchKernelGGL(bucket_mask_kernel, dim3((n_qb + MASK_BLOCKS_PER_WG - 1) / MASK_BLOCKS_PER_WG, H), dim3(256),
                       mask_lds, s, qbucket, n_q, m, (const int32_t *)nullptr, BQ, n_p, W, n_qb, qmask);
    FASTAR_LAUNCH_CHECK();
    hipLaunchKernelGGL(bucket_mask_kernel, dim3((n_kb_cap + MASK_BLOCKS_PER_WG - 1) / MASK_BLOCKS_PER_WG, H), dim3(256),
                       mask_lds, s, kbucket, C, m, len, BK, n_p, W, n_kb_cap, kmask);
    FASTAR_LAUNCH_CHECK();
    hipLaunchKernelGGL(bucket_score_kernel, dim3((n_kb_cap + 255) / 256, H), dim3(256), own_bytes, s, qmask, kmask, W,
                       n_qb, n_kb_cap, score);
    FASTAR_LAUNCH_CHECK();
    hipLaunchKernelGGL(bucket_topk_kernel, dim3(n_qb, H), dim3(256), (size_t)std::min(n_kb_cap, TOPK_LDS_CAP) * 4, s, score,
                       n_kb_cap, len, C, BK, n_qb, n_sel, n_sink, n_local, sel, nsel);
    FASTAR_LAUNCH_CHECK();
    return FASTAR_OK;
}
