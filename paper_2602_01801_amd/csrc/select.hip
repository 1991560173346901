// ANN selection (Sec. 5.1 goal "keys with the largest dot products"; Sec. 5.4 AnnSA; Sec. 5.3 AnnCA).
//
// Three stages, all on exact integer scores so that the selected sets are reproducible bit for bit:
//   rep_kernel          mean codes that summarise each query block (AnnSA only)
//   score_*_kernel      int8 matrix-core scoring of summaries x key codes, reduced on the fly to one
//                       int32 per (query block, key block) [AnnSA] or per (query block, prompt token)
//                       [AnnCA]; HBM-bound: every key code is streamed exactly once
//   topk                exact top-n_sel per row by radix select, ties to the lowest index, written in
//                       ascending order by ballot + prefix-sum compaction (a kernel of its own for AnnSA,
//                       the tail of the scoring kernel for AnnCA, where one workgroup owns a whole row)
#include <limits.h>

#include <algorithm>

#include "common.hpp"
#include "topk_dev.hpp"

namespace fastar {

constexpr int KB_PER_WG = 4;      // key blocks scored by one workgroup of score_self_kernel
constexpr size_t LONG_CACHE_BLOCKS = 16 * 4096;   // key blocks over all heads from which the streaming kernel pays
constexpr int COL_CHUNK = 8;       // summary column blocks (of 32) kept in registers at a time

static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// ---- codes narrower than a byte -----------------------------------------------------------------------
// Codes of BITS (2, 4 or 8) bits per entry, packed from the low end of each byte (appendix, "Quantization precision for
// ANN matching").  Key codes stay packed in memory and are widened in registers, as the matrix operand of one lane half
// (16 entries): an entry is moved to the TOP bits of its byte, i.e. multiplied by 2^(8-BITS) - the same factor on every
// score of a call, so no ranking changes - which needs one shift and one mask per four entries and no sign extension.
// Byte i of output word t then holds entry (8/BITS) * i' + t of its word; the summaries are stored in the same order.
template <int BITS>
__device__ __forceinline__ i32x4 load_key_codes(const int8_t *p) {   // p: the lane half's 16 * BITS / 8 bytes
    i32x4 a;
    if constexpr (BITS == 8) {
        a = *(const i32x4 *)p;
    } else if constexpr (BITS == 4) {
        const u32x2 w = *(const u32x2 *)p;
        a[0] = (int)((w[0] << 4) & 0xF0F0F0F0u);
        a[1] = (int)(w[0] & 0xF0F0F0F0u);
        a[2] = (int)((w[1] << 4) & 0xF0F0F0F0u);
        a[3] = (int)(w[1] & 0xF0F0F0F0u);
    } else {
        const unsigned w = *(const unsigned *)p;
        a[0] = (int)((w << 6) & 0xC0C0C0C0u);
        a[1] = (int)((w << 4) & 0xC0C0C0C0u);
        a[2] = (int)((w << 2) & 0xC0C0C0C0u);
        a[3] = (int)(w & 0xC0C0C0C0u);
    }
    return a;
}
// position, inside its group of 16, at which entry e of a summary is stored so that it meets the widened key entries
template <int BITS>
__device__ __forceinline__ int summary_slot(int e) {
    if constexpr (BITS == 8) return e;
    else if constexpr (BITS == 4) return (e & 8) + ((e & 1) << 2) + ((e & 7) >> 1);
    else return ((e & 3) << 2) + (e >> 2);
}

// ---- query-block summaries ------------------------------------------------------------------------
// rep[h][b*n_rep + u][j] = floor((sum over the u-th run of g queries of block b of qcode[.][j] + g/2) / g)
template <int BITS>
__global__ void rep_kernel(const int8_t *__restrict__ qcode, int n_q, int r, int BQ, int n_rep, int n_qb,
                           int8_t *__restrict__ rep) {
    const int b = blockIdx.x, h = blockIdx.y;
    const int g = BQ / n_rep;
    constexpr int PER = 8 / BITS;
    const int rb = r / PER;   // bytes per query row
    for (int t = threadIdx.x; t < n_rep * r; t += blockDim.x) {
        const int u = t / r, j = t % r;
        const int q0 = b * BQ + u * g;
        const int q1 = min(q0 + g, n_q);
        int s = 0;
        const int8_t *col = qcode + ((size_t)h * n_q + q0) * rb + j / PER;
        const int up = 32 - BITS * (j % PER + 1);   // shift that puts the entry at the top of a word, then arithmetic shift down
        const int n = q1 - q0;
        int q = 0;
        for (; q + 8 <= n; q += 8) {   // eight independent loads in flight
            int v[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = col[(size_t)(q + e) * rb];
#pragma unroll
            for (int e = 0; e < 8; ++e) s += BITS == 8 ? v[e] : ((int)((unsigned)v[e] << up) >> (32 - BITS));
        }
        for (; q < n; ++q) {
            const int v = col[(size_t)q * rb];
            s += BITS == 8 ? v : ((int)((unsigned)v << up) >> (32 - BITS));
        }
        s += g / 2;
        int m = s / g;
        if (s % g != 0 && s < 0) m -= 1;
        rep[((size_t)h * n_qb * n_rep + (size_t)b * n_rep + u) * r + (j & ~15) + summary_slot<BITS>(j & 15)] = (int8_t)m;
    }
}

// ---- AnnSA scoring -----------------------------------------------------------------------------------
// out[h][b][kb] = max over the summaries u of block b (whose run holds a query) and the live keys k of
// key block kb of rep[b,u] . kcode[k].   D = A x B with A rows = 32 keys, B columns = 32 summaries.
template <int R, int BITS>
__global__ __launch_bounds__(256) void score_self_kernel(const int8_t *__restrict__ kcode, const int32_t *__restrict__ len,
                                                         const int8_t *__restrict__ rep, int C, int n_q, int BQ,
                                                         int n_rep, int BK, int n_qb, int n_kb_cap,
                                                         int32_t *__restrict__ out) {
    constexpr int KS = R / 32;
    extern __shared__ int32_t tile[];  // [n_qb][KB_PER_WG]
    const int h = blockIdx.y;
    const int L = min(len[h], C);
    const int n_kb = (L + BK - 1) / BK;
    const int kb0 = blockIdx.x * KB_PER_WG;
    if (kb0 >= n_kb) return;  // whole workgroup beyond the live cache (uniform)
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int col = lane & 31, g2 = lane >> 5;
    const int NR = n_qb * n_rep;
    const int NCB = (NR + 31) / 32;
    const int g = BQ / n_rep;
    constexpr int RB = R * BITS / 8;   // bytes per key row
    const int8_t *kc = kcode + (size_t)h * C * RB;
    const int8_t *rp = rep + (size_t)h * NR * R;

    for (int cb0 = 0; cb0 < NCB; cb0 += COL_CHUNK) {
        i32x4 bfrag[COL_CHUNK][KS];
#pragma unroll
        for (int c = 0; c < COL_CHUNK; ++c) {
            const int rc = min((cb0 + c) * 32 + col, NR - 1);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) bfrag[c][ks] = *(const i32x4 *)(rp + (size_t)rc * R + ks * 32 + 16 * g2);
        }
        for (int kl = wave; kl < KB_PER_WG; kl += 4) {
            const int kb = kb0 + kl;
            if (kb >= n_kb) break;
            int best[COL_CHUNK];
#pragma unroll
            for (int c = 0; c < COL_CHUNK; ++c) best[c] = INT_MIN;
            // two groups of 32 keys per round: both loads are issued before the first product waits
            for (int sg0 = 0; sg0 < BK; sg0 += 64) {
                if (kb * BK + sg0 >= L) break;
                i32x4 afrag[2][KS];
                bool have[2], partial[2];
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const int sg = sg0 + 32 * q;
                    const int kbase = kb * BK + sg;
                    have[q] = sg < BK && kbase < L;
                    partial[q] = kbase + 32 > L || sg + 32 > BK;
                    const int krow = min(kbase + col, C - 1);
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) {
                        i32x4 a = {0, 0, 0, 0};
                        if (have[q]) a = load_key_codes<BITS>(kc + (size_t)krow * RB + (ks * 32 + 16 * g2) * BITS / 8);
                        afrag[q][ks] = a;
                    }
                }
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    if (!have[q]) continue;   // uniform
                    const int sg = sg0 + 32 * q;
                    const int kbase = kb * BK + sg;
#pragma unroll
                    for (int c = 0; c < COL_CHUNK; ++c) {
                        if (cb0 + c < NCB) {
                            i32x16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
                            for (int ks = 0; ks < KS; ++ks) acc = mfma_i8_32x32x32(afrag[q][ks], bfrag[c][ks], acc);
                            int m = best[c];
                            if (partial[q]) {
#pragma unroll
                                for (int v = 0; v < 16; ++v) {
                                    const int kloc = 8 * (v >> 2) + 4 * g2 + (v & 3);
                                    if (kbase + kloc < L && sg + kloc < BK) m = max(m, acc[v]);
                                }
                            } else {
#pragma unroll
                                for (int v = 0; v < 16; ++v) m = max(m, acc[v]);
                            }
                            best[c] = m;
                        }
                    }
                }
            }
#pragma unroll
            for (int c = 0; c < COL_CHUNK; ++c) {
                if (cb0 + c < NCB) {
                    int m = max(best[c], shfl_xor(best[c], 32));
                    const int rc = (cb0 + c) * 32 + col;
                    const int b = rc / n_rep, u = rc % n_rep;
                    if (rc >= NR || b * BQ + u * g >= n_q) m = INT_MIN;
                    for (int off = 1; off < n_rep; off <<= 1) m = max(m, shfl_xor(m, off));
                    if (g2 == 0 && u == 0 && rc < NR) tile[b * KB_PER_WG + kl] = m;
                }
            }
        }
    }
    __syncthreads();
    const int n_here = min(KB_PER_WG, n_kb - kb0);
    for (int t = threadIdx.x; t < n_qb * KB_PER_WG; t += blockDim.x) {
        const int b = t / KB_PER_WG, kl = t % KB_PER_WG;
        if (kl < n_here) out[((size_t)h * n_qb + b) * n_kb_cap + kb0 + kl] = tile[t];
    }
}

// Lane exchanges of the scoring epilogue without a trip through LDS.
__device__ __forceinline__ int max_across_halves_i32(int x) {   // max with lane ^ 32
    const auto r = __builtin_amdgcn_permlane32_swap((unsigned)x, (unsigned)x, false, false);
    return max((int)r[0], (int)r[1]);
}
__device__ __forceinline__ int max_over_quad_i32(int x) {       // max over the four lanes 4k .. 4k+3
    x = max(x, __builtin_amdgcn_update_dpp(x, x, 0xB1, 0xF, 0xF, false));   // quad_perm [1,0,3,2]
    return max(x, __builtin_amdgcn_update_dpp(x, x, 0x4E, 0xF, 0xF, false));   // quad_perm [2,3,0,1]
}

// The same scores for long caches.  What bounds this kernel is how the memory system is addressed: workgroups that
// each own a contiguous run of key blocks read at large, equal strides from each other and reach only about
// 2.8 TB/s on this chip, whatever they compute; workgroups that together sweep a dense window reach 5 TB/s and more.
// So the grid walks the head's key blocks in steps: in step s workgroup x takes blocks 4(sG + x) .. +3, one per
// wavefront, G = gridDim.x; a wavefront keeps the codes of its next three rounds in flight while it scores the current
// one (four operand buffers in an unrolled rotation: copying a buffer would wait for its loads) and writes its block's
// scores straight to the rows of the score matrix.  CC: summary column blocks (of 32) kept in registers at a time.
template <int R, int CC, int BITS>
__global__ __launch_bounds__(256, 3) void score_self_stream_kernel(const int8_t *__restrict__ kcode, const int32_t *__restrict__ len,
                                                         const int8_t *__restrict__ rep, int C, int n_q, int BQ,
                                                         int n_rep, int BK, int n_qb, int n_kb_cap,
                                                         int32_t *__restrict__ out) {
    constexpr int KS = R / 32;
    constexpr int RB = R * BITS / 8;   // bytes per key row
    const int h = blockIdx.y;
    const int L = min(len[h], C);
    const int n_kb = (L + BK - 1) / BK;
    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform, kept in a scalar register
    const int col = lane & 31, g2 = lane >> 5;
    const int NR = n_qb * n_rep;
    const int NCB = (NR + 31) / 32;
    const int g = BQ / n_rep;
    const int rep_shift = __ffs(n_rep) - 1;   // n_rep is a power of two
    const int8_t *kc = kcode + (size_t)h * C * RB;
    const int8_t *rp = rep + (size_t)h * NR * R;
    const int first = blockIdx.x * 4 + wave;          // this wavefront's first key block
    const int stride = gridDim.x * 4;                 // ... and the distance to its next one
    if (first >= n_kb) return;                        // nothing for this wavefront (no barrier follows)
    // rounds of 64 keys (two groups of 32): key block first + stride * (it / rpk), keys 64 * (it % rpk) .. of it
    const int rpk = (BK + 63) / 64;
    const int n_it = ((n_kb - first + stride - 1) / stride) * rpk;
    auto load_round = [&](int it, i32x4 (&a)[2][KS]) __attribute__((always_inline)) {
        it = min(it, n_it - 1);   // rounds past the wavefront's share re-read its last one (cache hits), never other blocks
        const int kb = first + stride * (it / rpk), sg0 = 64 * (it % rpk);
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int sg = sg0 + 32 * q;
            const int kbase = kb * BK + sg;
            // always loaded, from a clamped row: the number of loads in flight is then the same on every path and
            // the compiler can wait for exactly the buffer it needs; rows past the block or the cache are never scored
            const int krow = min(kbase + col, C - 1);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) a[q][ks] = load_key_codes<BITS>(kc + (size_t)krow * RB + (ks * 32 + 16 * g2) * BITS / 8);
        }
    };

    for (int cb0 = 0; cb0 < NCB; cb0 += CC) {
        i32x4 bfrag[CC][KS];
#pragma unroll
        for (int c = 0; c < CC; ++c) {
            const int rc = min((cb0 + c) * 32 + col, NR - 1);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) bfrag[c][ks] = *(const i32x4 *)(rp + (size_t)rc * R + ks * 32 + 16 * g2);
        }
        int best[CC];
        // what this lane's summary column of every column block stands for: its score row and whether it is the
        // block's first summary; columns past the summaries or of a run without a query never count
        int32_t *col_out[CC];
        bool col_ok[CC], col_first[CC];
#pragma unroll
        for (int c = 0; c < CC; ++c) {
            const int rc = (cb0 + c) * 32 + col;
            const int b = rc >> rep_shift;
            const int u = rc & (n_rep - 1);
            col_ok[c] = rc < NR && b * BQ + u * g < n_q;
            col_first[c] = rc < NR && u == 0 && g2 == 0;
            col_out[c] = out + ((size_t)h * n_qb + min(b, n_qb - 1)) * n_kb_cap;
        }
        const bool full_cols = cb0 + CC <= NCB;
        auto score_round = [&](int it, const i32x4 (&cur)[2][KS]) __attribute__((always_inline)) {
            if (it >= n_it) return;   // uniform
            const int kb = first + stride * (it / rpk), sg0 = 64 * (it % rpk);
            if (sg0 == 0) {
#pragma unroll
                for (int c = 0; c < CC; ++c) best[c] = INT_MIN;
            }
            if (full_cols && kb * BK + sg0 + 64 <= L && sg0 + 64 <= BK) {
                // the common round, straight line: 64 live keys, every column block in use
#pragma unroll
                for (int c = 0; c < CC; ++c) {
                    i32x16 acc0 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
                    i32x16 acc1 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) {
                        acc0 = mfma_i8_32x32x32(cur[0][ks], bfrag[c][ks], acc0);
                        acc1 = mfma_i8_32x32x32(cur[1][ks], bfrag[c][ks], acc1);
                    }
                    int m = best[c];
#pragma unroll
                    for (int v = 0; v < 16; ++v) m = max(max(m, acc0[v]), acc1[v]);   // one three-operand maximum each
                    best[c] = m;
                }
            } else {
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const int sg = sg0 + 32 * q;
                    const int kbase = kb * BK + sg;
                    if (!(sg < BK && kbase < L)) continue;   // uniform
                    const bool partial = kbase + 32 > L || sg + 32 > BK;
#pragma unroll
                    for (int c = 0; c < CC; ++c) {
                        if (cb0 + c < NCB) {
                            i32x16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
                            for (int ks = 0; ks < KS; ++ks) acc = mfma_i8_32x32x32(cur[q][ks], bfrag[c][ks], acc);
                            int m = best[c];
                            if (partial) {
#pragma unroll
                                for (int v = 0; v < 16; ++v) {
                                    const int kloc = 8 * (v >> 2) + 4 * g2 + (v & 3);
                                    if (kbase + kloc < L && sg + kloc < BK) m = max(m, acc[v]);
                                }
                            } else {
#pragma unroll
                                for (int v = 0; v < 16; ++v) m = max(m, acc[v]);
                            }
                            best[c] = m;
                        }
                    }
                }
            }
            if (it % rpk == rpk - 1) {   // the key block is complete
#pragma unroll
                for (int c = 0; c < CC; ++c) {
                    if (cb0 + c < NCB) {
                        int m = max_across_halves_i32(best[c]);
                        if (!col_ok[c]) m = INT_MIN;
                        if (n_rep == 4) m = max_over_quad_i32(m);   // uniform
                        else for (int off = 1; off < n_rep; off <<= 1) m = max(m, shfl_xor(m, off));
                        if (col_first[c]) col_out[c][kb] = m;
                    }
                }
            }
        };
        i32x4 b0[2][KS], b1[2][KS], b2[2][KS], b3[2][KS];
        load_round(0, b0);
        load_round(1, b1);
        load_round(2, b2);
        for (int it = 0; it < n_it; it += 4) {
            load_round(it + 3, b3);
            score_round(it, b0);
            load_round(it + 4, b0);
            score_round(it + 1, b1);
            load_round(it + 5, b1);
            score_round(it + 2, b2);
            load_round(it + 6, b2);
            score_round(it + 3, b3);
        }
    }
}

// ---- AnnCA scoring -----------------------------------------------------------------------------------
// score[p] = max over the queries q of block b of qcode[q] . pcode[p], kept in LDS, then the top n_sel of the row.
// D = A x B with A rows = 32 queries, B columns = 32 prompt tokens.
// smax[p] = max over the queries of block b of qcode[q] . pcode[p], for all n_p prompt tokens; whole workgroup.
template <int R>
__device__ __forceinline__ void score_cross_block(const int8_t *__restrict__ qc, const int8_t *__restrict__ pc, int n_q,
                                                  int n_p, int BQ, int b, int32_t *smax) {
    constexpr int KS = R / 32;
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int col = lane & 31, g2 = lane >> 5;
    for (int t = threadIdx.x; t < n_p; t += blockDim.x) smax[t] = INT_MIN;
    __syncthreads();
    const int q_end = min((b + 1) * BQ, n_q);
    for (int qg = b * BQ + wave * 32; qg < q_end; qg += 4 * 32) {
        const int qrow = min(qg + col, n_q - 1);
        i32x4 afrag[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) afrag[ks] = *(const i32x4 *)(qc + (size_t)qrow * R + ks * 32 + 16 * g2);
        const bool partial = qg + 32 > q_end;
        // eight groups of 32 prompt tokens per step: their codes are loaded together, then scored
        constexpr int PB = 8;
        for (int pb = 0; pb < n_p; pb += 32 * PB) {
            i32x4 bfrag[PB][KS];
#pragma unroll
            for (int u = 0; u < PB; ++u) {
                const int prow = min(pb + 32 * u + col, n_p - 1);
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) bfrag[u][ks] = *(const i32x4 *)(pc + (size_t)prow * R + ks * 32 + 16 * g2);
            }
#pragma unroll
            for (int u = 0; u < PB; ++u) {
                const int p0 = pb + 32 * u;
                if (p0 >= n_p) break;   // uniform
                i32x16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) acc = mfma_i8_32x32x32(afrag[ks], bfrag[u][ks], acc);
                int m = INT_MIN;
                if (partial) {
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        if (qg + 8 * (v >> 2) + 4 * g2 + (v & 3) < q_end) m = max(m, acc[v]);
                } else {
#pragma unroll
                    for (int v = 0; v < 16; ++v) m = max(m, acc[v]);
                }
                m = max(m, shfl_xor(m, 32));
                if (g2 == 0 && p0 + col < n_p) atomicMax(&smax[p0 + col], m);
            }
        }
    }
    __syncthreads();
}

template <int R>
__global__ __launch_bounds__(256) void score_cross_kernel(const int8_t *__restrict__ qcode, const int8_t *__restrict__ pcode,
                                                          int n_q, int n_p, int BQ, int n_qb, int n_sel,
                                                          int32_t *__restrict__ sel, int32_t *__restrict__ nsel) {
    extern __shared__ int32_t smax[];  // [n_p]
    const int b = blockIdx.x, h = blockIdx.y;
    score_cross_block<R>(qcode + (size_t)h * n_q * R, pcode + (size_t)h * n_p * R, n_q, n_p, BQ, b, smax);
    // the workgroup owns the whole row: select from LDS right away
    topk_row(smax, n_p, n_sel, sel + ((size_t)h * n_qb + b) * n_sel, nsel + (size_t)h * n_qb + b, nullptr);
}

// ---- AnnCA in one launch: selection and the attention over it (bf16, d = 128, blocks of 128 queries, up to 64 tokens) --
// One workgroup = one query block: scores and exact top-n_sel as above (the list also goes to sel / nsel), then the
// selected prompt rows are gathered into LDS once and the four wavefronts (32 queries each) attend to them:
// S^T = K Q^T, softmax over the at most 64 tokens in one piece (no running maximum), O^T = V^T P^T.  V is stored
// transposed ([d][token]) with the tokens of each 16 in the order the score accumulators hold them, so that the
// accumulators, converted to bf16, are the second product's operand as they are.
namespace fused {
constexpr int D = 128, TK = 64;
constexpr int KROW = D * 2 + 16;          // bytes per staged K row (padded: 16 consecutive rows hit 16 different bank groups)
constexpr int VROW = TK * 2 + 16;         // bytes per staged V^T row
constexpr int OROW = D * 2 + 16;          // bytes per staged output row
constexpr int TILE_BYTES = TK * KROW + D * VROW;   // 17408 + 18432; the output staging (128 rows x OROW) reuses it
static_assert(128 * OROW <= TILE_BYTES, "output staging fits the tile region");
__host__ __device__ inline size_t lds_bytes(int n_p) { return ((size_t)n_p * 4 + 15) / 16 * 16 + TK * 4 + 16 + TILE_BYTES; }
}  // namespace fused

template <int R>
__global__ __launch_bounds__(256) void cross_fused_kernel(const unsigned short *__restrict__ Q, const int8_t *__restrict__ qcode,
                                                          const unsigned short *__restrict__ Kp,
                                                          const unsigned short *__restrict__ Vp,
                                                          const int8_t *__restrict__ pcode, int n_q, int n_p, int n_qb,
                                                          int n_sel, float scale_log2, int32_t *__restrict__ sel,
                                                          int32_t *__restrict__ nsel, unsigned short *__restrict__ O) {
    using namespace fused;
    extern __shared__ __attribute__((aligned(16))) unsigned char flds[];
    int32_t *smax = (int32_t *)flds;
    int32_t *lsel = (int32_t *)(flds + ((size_t)n_p * 4 + 15) / 16 * 16);   // [TK] selected tokens, ascending
    int32_t *lcnt = lsel + TK;                                              // [1] how many
    unsigned char *ktile = (unsigned char *)(lcnt + 4);
    unsigned char *vtile = ktile + TK * KROW;
    const int b = blockIdx.x, h = blockIdx.y;
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const int col = lane & 31, g = lane >> 5;
    // this lane's query row as the second operand of K Q^T: in flight during the selection
    const int q_idx = b * 128 + wave * 32 + col;
    bf16x8 qf[D / 16];
    {
        const unsigned short *qrow = Q + ((size_t)h * n_q + min(q_idx, n_q - 1)) * D;
#pragma unroll
        for (int s = 0; s < D / 16; ++s) qf[s] = *(const bf16x8 *)(qrow + 16 * s + 8 * g);
    }
    score_cross_block<R>(qcode + (size_t)h * n_q * R, pcode + (size_t)h * n_p * R, n_q, n_p, 128, b, smax);
    topk_row(smax, n_p, n_sel, lsel, lcnt, nullptr);
    __syncthreads();
    const int k = lcnt[0];
    if (tid < n_sel) sel[((size_t)h * n_qb + b) * n_sel + tid] = lsel[tid];
    if (tid == 0) nsel[(size_t)h * n_qb + b] = k;
    // gather: K rows as they are, V rows transposed; slot p of the tile holds token lsel[p] (p >= k: token 0, masked below)
    const unsigned short *Kh = Kp + (size_t)h * n_p * D, *Vh = Vp + (size_t)h * n_p * D;
    {
        u32x4 kv[4], vv[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int idx = e * 256 + tid, p = idx >> 4, c = idx & 15;
            const int tok = p < k ? lsel[p] : 0;
            kv[e] = *(const u32x4 *)(Kh + (size_t)tok * D + 8 * c);
            vv[e] = *(const u32x4 *)(Vh + (size_t)tok * D + 8 * c);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int idx = e * 256 + tid, p = idx >> 4, c = idx & 15;
            *(u32x4 *)(ktile + p * KROW + c * 16) = kv[e];
            // position of token slot p inside its 16: accumulator order (half g' = (o % 8) / 4 first, then o / 8, then o % 4)
            const int o = p & 15;
            const int pos = (p & ~15) + 8 * ((o & 7) >> 2) + 4 * (o >> 3) + (o & 3);
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                *(unsigned short *)(vtile + (8 * c + 2 * w) * VROW + pos * 2) = (unsigned short)(vv[e][w] & 0xFFFFu);
                *(unsigned short *)(vtile + (8 * c + 2 * w + 1) * VROW + pos * 2) = (unsigned short)(vv[e][w] >> 16);
            }
        }
    }
    __syncthreads();
    // S^T = K Q^T: rows = token slots (two blocks of 32), columns = this wavefront's 32 queries
    f32x16 s_acc[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
        for (int v = 0; v < 16; ++v) s_acc[kb][v] = 0.0f;
#pragma unroll
        for (int s = 0; s < D / 16; ++s) {
            const bf16x8 a = *(const bf16x8 *)(ktile + (32 * kb + col) * KROW + (16 * s + 8 * g) * 2);
            s_acc[kb] = mfma_bf16_32x32x16(a, qf[s], s_acc[kb]);
        }
    }
    // softmax over the k live slots (register v of block kb is slot 32 kb + 8 (v / 4) + 4 g + v % 4)
    float mx = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int slot = 32 * kb + 8 * (v >> 2) + 4 * g + (v & 3);
            if (slot >= k) s_acc[kb][v] = -INFINITY;
            mx = fmaxf(mx, s_acc[kb][v]);
        }
    mx = fmaxf(mx, shfl_xor(mx, 32));
    const float neg_ms = mx == -INFINITY ? 0.0f : -mx * scale_log2;
    float l = 0.0f;
    bf16x8 pf[2][2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int st = 0; st < 2; ++st)
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float pv = __builtin_amdgcn_exp2f(fmaf(s_acc[kb][8 * st + j], scale_log2, neg_ms));
                const __bf16 pb = (__bf16)pv;
                pf[kb][st][j] = pb;
                l += (float)pb;   // the sum takes the rounded P, the values the second product sees
            }
    l += shfl_xor(l, 32);
    // O^T = V^T P^T: rows = 32 of the d coordinates per block, columns = queries
    f32x16 o_acc[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db) {
#pragma unroll
        for (int v = 0; v < 16; ++v) o_acc[db][v] = 0.0f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int st = 0; st < 2; ++st) {
                const bf16x8 a = *(const bf16x8 *)(vtile + (32 * db + col) * VROW + (32 * kb + 16 * st + 8 * g) * 2);
                o_acc[db] = mfma_bf16_32x32x16(a, pf[kb][st], o_acc[db]);
            }
    }
    const float inv = l > 0.0f ? 1.0f / l : 0.0f;
    __syncthreads();   // the tiles are dead: their LDS takes the output rows
    unsigned char *orow = ktile + (size_t)(wave * 32 + col) * OROW;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            u32x2 w;
            w[0] = pack_bf16x2(o_acc[db][4 * q4] * inv, o_acc[db][4 * q4 + 1] * inv);
            w[1] = pack_bf16x2(o_acc[db][4 * q4 + 2] * inv, o_acc[db][4 * q4 + 3] * inv);
            *(u32x2 *)(orow + (32 * db + 8 * q4 + 4 * g) * 2) = w;
        }
    __syncthreads();
    for (int idx = tid; idx < 128 * 16; idx += 256) {
        const int r = idx >> 4, c = idx & 15;
        const int qi = b * 128 + r;
        if (qi < n_q) *(u32x4 *)(O + ((size_t)h * n_q + qi) * D + 8 * c) = *(const u32x4 *)(ktile + (size_t)r * OROW + c * 16);
    }
}

// Row (h, b) of `score` holds n entries (n = ceil(len[h]/BK) when len is given, else n_fixed).
__global__ __launch_bounds__(256) void topk_kernel(const int32_t *__restrict__ score, int row_stride,
                                                   const int32_t *__restrict__ len, int len_cap, int BK, int n_fixed,
                                                   int n_qb, int n_sel, int32_t *__restrict__ sel,
                                                   int32_t *__restrict__ nsel, int n_sink, int n_local, int cand_min) {
    // staging of the row's keys: min(row_stride, TOPK_LDS_CAP) words of dynamic LDS (a static array of the full size
    // would hold the kernel to four workgroups per compute unit whatever the row length)
    extern __shared__ unsigned keys[];
    const int b = blockIdx.x, h = blockIdx.y;
    int n = n_fixed;
    if (len) n = (min(len[h], len_cap) + BK - 1) / BK;
    n = min(n, row_stride);
    const int32_t *row = score + ((size_t)h * n_qb + b) * row_stride;
    // cand_min > INT_MIN: only entries that score at least that much (or are forced) may be selected
    const int k_cap = cand_min > INT_MIN ? count_candidates(row, n, n_sink, n_local, cand_min) : INT_MAX;
    topk_row(row, n, n_sel, sel + ((size_t)h * n_qb + b) * n_sel, nsel + (size_t)h * n_qb + b, keys, n_sink, n_local,
             k_cap);
}

// ---- selection on sign codes (LSH family) -------------------------------------------------------------
// Summaries: bit j of the summary of a run of g queries = majority of the run's bits (2 * ones >= queries).
// One workgroup per (query block, head), one thread per hash bit; a wavefront's ballot is two words.
__global__ __launch_bounds__(256) void lsh_summary_kernel(const uint32_t *__restrict__ qbits, int n_q, int W, int BQ,
                                                          int n_rep, int n_qb, uint32_t *__restrict__ rep) {
    extern __shared__ uint32_t qw[];  // the query block's codes, [BQ][W]
    const int b = blockIdx.x, h = blockIdx.y, j = threadIdx.x;
    const int g = BQ / n_rep;
    const int lane = lane_id(), wave = j >> 6;
    const bool mine = j < 32 * W;
    const int q_lo = b * BQ, q_hi = min(q_lo + BQ, n_q);
    // one round of loads for the whole block, then the votes are counted from LDS
    for (int t = j; t < (q_hi - q_lo) * W; t += blockDim.x) qw[t] = qbits[((size_t)h * n_q + q_lo) * W + t];
    __syncthreads();
    for (int u = 0; u < n_rep; ++u) {
        const int q0 = q_lo + u * g, q1 = min(q0 + g, n_q);
        int ones = 0;
        if (mine)
            for (int q = q0; q < q1; ++q) ones += (int)((qw[(q - q_lo) * W + (j >> 5)] >> (j & 31)) & 1u);
        const unsigned long long m = __ballot(mine && q1 > q0 && 2 * ones >= q1 - q0);
        uint32_t *out = rep + ((size_t)h * n_qb * n_rep + (size_t)b * n_rep + u) * W;
        if (lane == 0 && 2 * wave < W) out[2 * wave] = (uint32_t)m;
        if (lane == 0 && 2 * wave + 1 < W) out[2 * wave + 1] = (uint32_t)(m >> 32);
    }
}

// out[h][b][kb] = max over the summaries u of block b (whose run holds a query) and the live keys k of key block
// kb of the number of equal bits.  A lane owns one key (its W words in registers) and walks all summaries (the
// same for every lane: scalar loads); the maximum over a key block is a reduction over BK lanes (BK a power of two
// <= 64) or over several 64-key rounds of a wavefront (BK a multiple of 64).
constexpr int LSH_QB = 8;  // query blocks whose scores a lane carries at a time

// Score of one 32-bit word of a (summary, key) pair, d = summary ^ key.
// BAND = 0: equal bits.  BAND in {4, 8, 16, 32}: the word holds 32/BAND hash tables (bands); a table counts when the
// two buckets differ in at most `radius` bits (0: same bucket; more: the neighbouring buckets are probed too).  Bits
// set per band by the usual pairwise sums, then one add per word whose carry into each band's top bit says "more than
// radius"; rc = that addend (see lsh_radius_addend).
template <int BAND>
__device__ __forceinline__ int lsh_word_score(unsigned d, unsigned rc, int radius) {
    if constexpr (BAND == 0) {
        return __popc(~d);
    } else {
        unsigned c = d - ((d >> 1) & 0x55555555u);
        c = (c & 0x33333333u) + ((c >> 2) & 0x33333333u);
        if constexpr (BAND == 4) return 8 - __popc((c + rc) & 0x88888888u);
        c = (c + (c >> 4)) & 0x0F0F0F0Fu;
        if constexpr (BAND == 8) return 4 - __popc((c + rc) & 0x80808080u);
        c = (c + (c >> 8)) & 0x00FF00FFu;
        if constexpr (BAND == 16) return 2 - __popc((c + rc) & 0x80008000u);
        c = (c + (c >> 16)) & 0xFFFFu;
        return (int)c <= radius ? 1 : 0;
    }
}
static inline unsigned lsh_radius_addend(int band, int radius) {
    if (band == 4) return (unsigned)(7 - radius) * 0x11111111u;
    if (band == 8) return (unsigned)(0x7F - radius) * 0x01010101u;
    if (band == 16) return (unsigned)(0x7FFF - radius) * 0x00010001u;
    return 0u;
}

template <int W, int BAND>
__global__ __launch_bounds__(256) void lsh_score_kernel(const uint32_t *__restrict__ kbits, const int32_t *__restrict__ len,
                                                        const uint32_t *__restrict__ rep, int C, int n_q, int BQ,
                                                        int n_rep, int BK, int n_qb, int n_kb_cap, int lds_words,
                                                        unsigned rc, int radius, int32_t *__restrict__ out) {
    const int h = blockIdx.y;
    const int L = min(len[h], C);
    const int n_kb = (L + BK - 1) / BK;
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int g = BQ / n_rep;
    const uint32_t *kb_h = kbits + (size_t)h * C * W;
    const uint32_t *rp = rep + (size_t)h * n_qb * n_rep * W;
    // the head's summaries are staged in LDS when they fit (lds_words > 0): every lane reads the same word
    extern __shared__ uint32_t srep[];
    if (lds_words > 0) {
        for (int t = threadIdx.x; t < lds_words; t += blockDim.x) srep[t] = rp[t];
        __syncthreads();
        rp = srep;
    }
    const int rounds = BK > 64 ? BK / 64 : 1;             // 64-key rounds per key block
    const int kb_per_round = BK >= 64 ? 1 : 64 / BK;      // key blocks covered by one round of 64 lanes
    // unit = one round-set: kb_per_round key blocks (BK < 64) or one key block (BK >= 64)
    const int n_units = (n_kb + kb_per_round - 1) / kb_per_round;
    for (int unit = blockIdx.x * 4 + wave; unit < n_units; unit += gridDim.x * 4) {
        uint32_t kw[W];   // this lane's key when a key block fits one round (re-read per round otherwise)
        bool live = false;
        if (rounds == 1) {
            const int key = BK >= 64 ? unit * BK + lane : unit * 64 + lane;
            live = key < L;
#pragma unroll
            for (int w = 0; w < W; ++w) kw[w] = live ? kb_h[(size_t)key * W + w] : 0u;
        }
        // query blocks in batches of LSH_QB: the lane-exchange reductions of a batch are independent of each other
        for (int b0 = 0; b0 < n_qb; b0 += LSH_QB) {
            int best[LSH_QB];
#pragma unroll
            for (int i = 0; i < LSH_QB; ++i) best[i] = -1;
            for (int rd = 0; rd < rounds; ++rd) {
                if (rounds > 1) {
                    const int key = unit * BK + rd * 64 + lane;
                    live = key < L;
#pragma unroll
                    for (int w = 0; w < W; ++w) kw[w] = live ? kb_h[(size_t)key * W + w] : 0u;
                }
#pragma unroll
                for (int i = 0; i < LSH_QB; ++i) {
                    const int b = b0 + i;
                    if (b >= n_qb) break;  // uniform
                    for (int u = 0; u < n_rep; ++u) {
                        if (b * BQ + u * g >= n_q) break;  // uniform: this run and the later ones hold no query
                        const uint32_t *r = rp + ((size_t)b * n_rep + u) * W;
                        int eq = 0;
#pragma unroll
                        for (int w = 0; w < W; ++w) eq += lsh_word_score<BAND>(r[w] ^ kw[w], rc, radius);
                        if (live) best[i] = max(best[i], eq);
                    }
                }
            }
            // maximum over the lanes of a key block
            const int span = BK >= 64 ? 64 : BK;
            for (int off = 1; off < span; off <<= 1) {
#pragma unroll
                for (int i = 0; i < LSH_QB; ++i) best[i] = max(best[i], shfl_xor(best[i], off));
            }
            const int kb = BK >= 64 ? unit : unit * kb_per_round + lane / BK;
            if ((lane & (span - 1)) == 0 && kb < n_kb) {
#pragma unroll
                for (int i = 0; i < LSH_QB; ++i)
                    if (b0 + i < n_qb) out[((size_t)h * n_qb + b0 + i) * n_kb_cap + kb] = best[i];
            }
        }
    }
}

struct LshWs {
    size_t rep_off, score_off, total;
};
static LshWs lsh_ws(int H, int n_q, int C, int n_bits, int BQ, int BK, int n_rep) {
    const int n_qb = (n_q + BQ - 1) / BQ;
    const int n_kb_cap = (C + BK - 1) / BK;
    LshWs w;
    w.rep_off = 0;
    w.score_off = align256((size_t)H * n_qb * n_rep * (n_bits / 8));
    w.total = w.score_off + align256((size_t)H * n_qb * n_kb_cap * sizeof(int32_t));
    return w;
}
size_t select_lsh_ws_bytes(int H, int n_q, int C, int n_bits, int BQ, int BK, int n_rep) {
    if (H <= 0 || n_q <= 0 || C <= 0 || n_bits <= 0 || BQ <= 0 || BK <= 0 || n_rep <= 0) return 0;
    return lsh_ws(H, n_q, C, n_bits, BQ, BK, n_rep).total;
}

static bool pow2_le32(int v) { return v >= 1 && v <= 32 && (v & (v - 1)) == 0; }

struct SelfWs {
    size_t rep_off, score_off, total;
};
static SelfWs self_ws(int H, int n_q, int C, int r, int BQ, int BK, int n_rep) {
    const int n_qb = (n_q + BQ - 1) / BQ;
    const int n_kb_cap = (C + BK - 1) / BK;
    SelfWs w;
    w.rep_off = 0;
    w.score_off = align256((size_t)H * n_qb * n_rep * r);
    w.total = w.score_off + align256((size_t)H * n_qb * n_kb_cap * sizeof(int32_t));
    return w;
}

size_t select_self_ws_bytes(int H, int n_q, int C, int r, int BQ, int BK, int n_rep) {
    if (H <= 0 || n_q <= 0 || C <= 0 || r <= 0 || BQ <= 0 || BK <= 0 || n_rep <= 0) return 0;
    return self_ws(H, n_q, C, r, BQ, BK, n_rep).total;
}
size_t select_cross_ws_bytes(int H, int n_q, int n_p, int BQ) {
    if (H <= 0 || n_q <= 0 || n_p <= 0 || BQ <= 0) return 0;
    const int n_qb = (n_q + BQ - 1) / BQ;
    return align256((size_t)H * n_qb * n_p * sizeof(int32_t));
}

int static_scratch_setup();

// more than 64 KB of LDS (long prompts) has to be allowed once per kernel and device; fastar_init also resolves the
// static scratch through this
int select_setup() {
    if (const int rc = static_scratch_setup(); rc != FASTAR_OK) return rc;
    static DeviceOnce once;
    return once.run([](int) {
        if (hipFuncSetAttribute((const void *)cross_fused_kernel<32>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)fused::lds_bytes(12288)) != hipSuccess ||
            hipFuncSetAttribute((const void *)cross_fused_kernel<64>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)fused::lds_bytes(12288)) != hipSuccess)
            return FASTAR_ERR_HIP;
        return FASTAR_OK;
    });
}

}  // namespace fastar

using namespace fastar;

static int select_self_impl(const int8_t *qcode, int n_q, const int8_t *kcode, const int32_t *len, int H, int C, int r,
                            int BQ, int n_rep, int BK, int n_sel, int32_t *sel, int32_t *nsel, void *ws,
                            size_t ws_bytes, void *stream, int n_sink = 0, int n_local = 0, int bits = 8) {
    if (!qcode || !kcode || !len || !sel || !nsel || !ws) return FASTAR_ERR_INVALID_ARG;
    if (n_sink < 0 || n_local < 0 || n_sink + n_local > n_sel) return FASTAR_ERR_INVALID_ARG;
    if (H <= 0 || n_q <= 0 || C <= 0 || BQ <= 0 || n_rep <= 0 || BK <= 0 || n_sel <= 0) return FASTAR_ERR_INVALID_ARG;
    if (BQ % n_rep != 0) return FASTAR_ERR_INVALID_ARG;
    if (((uintptr_t)qcode & 15) || ((uintptr_t)kcode & 15) || ((uintptr_t)ws & 255)) return FASTAR_ERR_INVALID_ARG;
    if ((r != 32 && r != 64) || !pow2_le32(n_rep) || BK % 32 != 0) return FASTAR_ERR_UNSUPPORTED;
    if (bits != 8 && !((bits == 4 || bits == 2) && r == 32)) return FASTAR_ERR_UNSUPPORTED;
    const int n_qb = (n_q + BQ - 1) / BQ;
    const int n_kb_cap = (C + BK - 1) / BK;
    // long caches whose summaries fit four column blocks take the streaming kernel: about 2048 workgroups that
    // sweep each head's key blocks together
    const bool few_cols = (n_qb * n_rep + 31) / 32 <= 4;
    const bool stream_kernel = few_cols && (size_t)n_kb_cap * H >= LONG_CACHE_BLOCKS;
    const size_t tile_bytes = (size_t)n_qb * KB_PER_WG * sizeof(int32_t);
    if (!stream_kernel && tile_bytes > 64 * 1024) return FASTAR_ERR_UNSUPPORTED;
    const SelfWs w = self_ws(H, n_q, C, r, BQ, BK, n_rep);
    if (ws_bytes < w.total) return FASTAR_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    int8_t *rep = (int8_t *)ws + w.rep_off;
    int32_t *score = (int32_t *)((char *)ws + w.score_off);
    const dim3 grid((n_kb_cap + KB_PER_WG - 1) / KB_PER_WG, H);
    constexpr int stream_wgs = 768;   // three resident workgroups per CU (the kernel is built for 168 registers)
    const dim3 grid_stream((unsigned)std::max(1, std::min(std::max(1, stream_wgs / H), (n_kb_cap + 3) / 4)), H);
#define FASTAR_SELF(RR, BB)                                                                                            \
    do {                                                                                                               \
        hipLaunchKernelGGL(rep_kernel<BB>, dim3(n_qb, H), dim3(128), 0, s, qcode, n_q, r, BQ, n_rep, n_qb, rep);       \
        FASTAR_LAUNCH_CHECK();                                                                                         \
        if (!stream_kernel)                                                                                            \
            hipLaunchKernelGGL((score_self_kernel<RR, BB>), grid, dim3(256), tile_bytes, s, kcode, len, rep, C, n_q, BQ, \
                               n_rep, BK, n_qb, n_kb_cap, score);                                                      \
        else                                                                                                           \
            hipLaunchKernelGGL((score_self_stream_kernel<RR, 4, BB>), grid_stream, dim3(256), 0, s, kcode, len, rep, C, \
                               n_q, BQ, n_rep, BK, n_qb, n_kb_cap, score);                                             \
    } while (0)
    if (bits == 4) FASTAR_SELF(32, 4);
    else if (bits == 2) FASTAR_SELF(32, 2);
    else if (r == 32) FASTAR_SELF(32, 8);
    else FASTAR_SELF(64, 8);
#undef FASTAR_SELF
    FASTAR_LAUNCH_CHECK();
    hipLaunchKernelGGL(topk_kernel, dim3(n_qb, H), dim3(256), (size_t)std::min(n_kb_cap, TOPK_LDS_CAP) * 4, s, score, n_kb_cap,
                       len, C, BK, 0, n_qb, n_sel, sel, nsel, n_sink, n_local, INT_MIN);
    FASTAR_LAUNCH_CHECK();
    return FASTAR_OK;
}

extern "C" int ann_select_self(const int8_t *qcode, int n_q, const int8_t *kcode, const int32_t *len, int H, int C,
                               int r, int BQ, int n_rep, int BK, int n_sel, int32_t *sel, int32_t *nsel, void *ws,
                               size_t ws_bytes, void *stream) {
    return select_self_impl(qcode, n_q, kcode, len, H, C, r, BQ, n_rep, BK, n_sel, sel, nsel, ws, ws_bytes, stream);
}

extern "C" int ann_select_self_forced(const int8_t *qcode, int n_q, const int8_t *kcode, const int32_t *len, int H,
                                      int C, int r, int BQ, int n_rep, int BK, int n_sel, int n_sink, int n_local,
                                      int32_t *sel, int32_t *nsel, void *ws, size_t ws_bytes, void *stream) {
    return select_self_impl(qcode, n_q, kcode, len, H, C, r, BQ, n_rep, BK, n_sel, sel, nsel, ws, ws_bytes, stream, n_sink,
                            n_local);
}

extern "C" int ann_select_self_packed(const int8_t *qcode, int n_q, const int8_t *kcode, const int32_t *len, int H,
                                      int C, int r, int bits, int BQ, int n_rep, int BK, int n_sel, int n_sink,
                                      int n_local, int32_t *sel, int32_t *nsel, void *ws, size_t ws_bytes, void *stream) {
    if (bits != 2 && bits != 4 && bits != 8) return FASTAR_ERR_INVALID_ARG;
    return select_self_impl(qcode, n_q, kcode, len, H, C, r, BQ, n_rep, BK, n_sel, sel, nsel, ws, ws_bytes, stream, n_sink,
                            n_local, bits);
}

// ---- the same selection on the library's own static scratch, for callers that cannot allocate ----------------------
// `scratch` is device memory that every GPU the library runs on holds until the process ends.  In host code the name
// is only a stand-in for the symbol: the device address is looked up once per device (with that device current) and
// kept; kernels, and anything else on the host that needs the memory, use that pointer.
static __device__ __align__(256) unsigned char scratch[FASTAR_STATIC_SCRATCH_BYTES];
static void *scratch_ptr[DeviceOnce::MAX_DEVICES];

namespace fastar {
int static_scratch_setup() {
    static DeviceOnce once;
    return once.run([](int dev) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return FASTAR_ERR_HIP;
        scratch_ptr[dev] = p;
        return FASTAR_OK;
    });
}
}  // namespace fastar

extern "C" int ann_select_self_static(const int8_t *qcode, int n_q, const int8_t *kcode, const int32_t *len, int H,
                                      int C, int r, int BQ, int n_rep, int BK, int n_sel, int32_t *sel, int32_t *nsel,
                                      void *stream) {
    if (H <= 0 || n_q <= 0 || C <= 0 || r <= 0 || BQ <= 0 || n_rep <= 0 || BK <= 0) return FASTAR_ERR_INVALID_ARG;
    if (self_ws(H, n_q, C, r, BQ, BK, n_rep).total > (size_t)FASTAR_STATIC_SCRATCH_BYTES) return FASTAR_ERR_STATIC_SCRATCH;
    if (const int rc = static_scratch_setup(); rc != FASTAR_OK) return rc;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return FASTAR_ERR_HIP;
    // nothing in the scratch has to start from zero: the summaries and every score row that the top-k reads are
    // written by this call's own launches before they are read
    return select_self_impl(qcode, n_q, kcode, len, H, C, r, BQ, n_rep, BK, n_sel, sel, nsel, scratch_ptr[dev],
                            (size_t)FASTAR_STATIC_SCRATCH_BYTES, stream);
}

extern "C" int ann_select_cross(const int8_t *qcode, int n_q, const int8_t *pcode, int n_p, int H, int r, int BQ,
                                int n_sel, int32_t *sel, int32_t *nsel, void *ws, size_t ws_bytes, void *stream) {
    if (!qcode || !pcode || !sel || !nsel || !ws) return FASTAR_ERR_INVALID_ARG;
    if (H <= 0 || n_q <= 0 || n_p <= 0 || BQ <= 0 || n_sel <= 0) return FASTAR_ERR_INVALID_ARG;
    if (((uintptr_t)qcode & 15) || ((uintptr_t)pcode & 15) || ((uintptr_t)ws & 255)) return FASTAR_ERR_INVALID_ARG;
    if ((r != 32 && r != 64) || n_p > 12288) return FASTAR_ERR_UNSUPPORTED;
    const int n_qb = (n_q + BQ - 1) / BQ;
    if (ws_bytes < select_cross_ws_bytes(H, n_q, n_p, BQ)) return FASTAR_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    const size_t lds = (size_t)n_p * sizeof(int32_t);
    if (r == 32)
        hipLaunchKernelGGL(score_cross_kernel<32>, dim3(n_qb, H), dim3(256), lds, s, qcode, pcode, n_q, n_p, BQ, n_qb,
                           n_sel, sel, nsel);
    else
        hipLaunchKernelGGL(score_cross_kernel<64>, dim3(n_qb, H), dim3(256), lds, s, qcode, pcode, n_q, n_p, BQ, n_qb,
                           n_sel, sel, nsel);
    FASTAR_LAUNCH_CHECK();
    return FASTAR_OK;
}

extern "C" int ann_cross_attn_fwd(const void *Q, const int8_t *qcode, int n_q, const void *Kp, const void *Vp,
                                  const int8_t *pcode, int n_p, int H, int d, int dtype, int r, int BQ, int n_sel,
                                  float scale, int32_t *sel, int32_t *nsel, void *O, void *stream) {
    if (!Q || !qcode || !Kp || !Vp || !pcode || !sel || !nsel || !O) return FASTAR_ERR_INVALID_ARG;
    if (H <= 0 || n_q <= 0 || n_p <= 0 || n_sel <= 0) return FASTAR_ERR_INVALID_ARG;
    if (!(scale > 0.0f) || !(scale < INFINITY)) return FASTAR_ERR_INVALID_ARG;
    if (((uintptr_t)Q & 15) || ((uintptr_t)Kp & 15) || ((uintptr_t)Vp & 15) || ((uintptr_t)O & 15) ||
        ((uintptr_t)qcode & 15) || ((uintptr_t)pcode & 15))
        return FASTAR_ERR_INVALID_ARG;
    if (dtype != FASTAR_BF16 || d != 128 || BQ != 128 || n_sel > fused::TK || (r != 32 && r != 64) || n_p > 12288)
        return FASTAR_ERR_UNSUPPORTED;
    const int n_qb = (n_q + 127) / 128;
    const size_t lds = fused::lds_bytes(n_p);
    hipStream_t s = (hipStream_t)stream;
    const float scale_log2 = scale * 1.4426950408889634f;
    if (const int rc = select_setup(); rc != FASTAR_OK) return rc;
    if (r == 32)
        hipLaunchKernelGGL(cross_fused_kernel<32>, dim3(n_qb, H), dim3(256), lds, s, (const unsigned short *)Q, qcode,
                           (const unsigned short *)Kp, (const unsigned short *)Vp, pcode, n_q, n_p, n_qb, n_sel,
                           scale_log2, sel, nsel, (unsigned short *)O);
    else
        hipLaunchKernelGGL(cross_fused_kernel<64>, dim3(n_qb, H), dim3(256), lds, s, (const unsigned short *)Q, qcode,
                           (const unsigned short *)Kp, (const unsigned short *)Vp, pcode, n_q, n_p, n_qb, n_sel,
                           scale_log2, sel, nsel, (unsigned short *)O);
    FASTAR_LAUNCH_CHECK();
    return FASTAR_OK;
}

static int select_lsh_impl(const uint32_t *qbits, int n_q, const uint32_t *kbits, const int32_t *len, int H, int C,
                           int n_bits, int band, int radius, int BQ, int n_rep, int BK, int n_sel, int n_sink, int n_local,
                           int32_t *sel, int32_t *nsel, void *ws, size_t ws_bytes, void *stream) {
    if (!qbits || !kbits || !len || !sel || !nsel || !ws) return FASTAR_ERR_INVALID_ARG;
    if (H <= 0 || n_q <= 0 || C <= 0 || BQ <= 0 || n_rep <= 0 || BK <= 0 || n_sel <= 0) return FASTAR_ERR_INVALID_ARG;
    if (BQ % n_rep != 0 || ((uintptr_t)ws & 255)) return FASTAR_ERR_INVALID_ARG;
    if (radius < 0 || n_sink < 0 || n_local < 0 || n_sink + n_local > n_sel) return FASTAR_ERR_INVALID_ARG;
    if (n_bits != 64 && n_bits != 128 && n_bits != 256) return FASTAR_ERR_UNSUPPORTED;
    if (band != 0 && band != 4 && band != 8 && band != 16 && band != 32) return FASTAR_ERR_UNSUPPORTED;
    if (!((BK <= 64 && (BK & (BK - 1)) == 0) || BK % 64 == 0)) return FASTAR_ERR_UNSUPPORTED;
    if (band && radius > band) radius = band;   // every bucket of a table is probed from there on
    const int W = n_bits / 32;
    const int n_qb = (n_q + BQ - 1) / BQ;
    const int n_kb_cap = (C + BK - 1) / BK;
    const LshWs w = lsh_ws(H, n_q, C, n_bits, BQ, BK, n_rep);
    if (ws_bytes < w.total) return FASTAR_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    uint32_t *rep = (uint32_t *)((char *)ws + w.rep_off);
    int32_t *score = (int32_t *)((char *)ws + w.score_off);
    if ((size_t)BQ * W * 4 > 48 * 1024) return FASTAR_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(lsh_summary_kernel, dim3(n_qb, H), dim3(256), (size_t)BQ * W * 4, s, qbits, n_q, W, BQ, n_rep, n_qb,
                       rep);
    FASTAR_LAUNCH_CHECK();
    const int kb_per_round = BK >= 64 ? 1 : 64 / BK;
    const int n_units = (n_kb_cap + kb_per_round - 1) / kb_per_round;
    dim3 grid((n_units + 3) / 4, H);
    int lds_words = n_qb * n_rep * W;
    if ((size_t)lds_words * 4 > 48 * 1024) lds_words = 0;  // too many summaries (per-query form): read them from memory
    const size_t lds_bytes = (size_t)lds_words * 4;
    const unsigned rc = lsh_radius_addend(band, radius);
#define FASTAR_LSH(WW, BB)                                                                                             \
    hipLaunchKernelGGL((lsh_score_kernel<WW, BB>), grid, dim3(256), lds_bytes, s, kbits, len, rep, C, n_q, BQ, n_rep, BK, \
                       n_qb, n_kb_cap, lds_words, rc, radius, score)
#define FASTAR_LSH_W(BB)                        \
    do {                                        \
        if (W == 2) FASTAR_LSH(2, BB);          \
        else if (W == 4) FASTAR_LSH(4, BB);     \
        else FASTAR_LSH(8, BB);                 \
    } while (0)
    if (band == 0) FASTAR_LSH_W(0);
    else if (band == 4) FASTAR_LSH_W(4);
    else if (band == 8) FASTAR_LSH_W(8);
    else if (band == 16) FASTAR_LSH_W(16);
    else FASTAR_LSH_W(32);
#undef FASTAR_LSH_W
#undef FASTAR_LSH
    FASTAR_LAUNCH_CHECK();
    // with tables only key blocks with a collision are candidates
    hipLaunchKernelGGL(topk_kernel, dim3(n_qb, H), dim3(256), (size_t)std::min(n_kb_cap, TOPK_LDS_CAP) * 4, s, score, n_kb_cap,
                       len, C, BK, 0, n_qb, n_sel, sel, nsel, n_sink, n_local, band ? 1 : INT_MIN);
    FASTAR_LAUNCH_CHECK();
    return FASTAR_OK;
}

extern "C" int ann_select_lsh(const uint32_t *qbits, int n_q, const uint32_t *kbits, const int32_t *len, int H, int C,
                              int n_bits, int BQ, int n_rep, int BK, int n_sel, int32_t *sel, int32_t *nsel, void *ws,
                              size_t ws_bytes, void *stream) {
    return select_lsh_impl(qbits, n_q, kbits, len, H, C, n_bits, 0, 0, BQ, n_rep, BK, n_sel, 0, 0, sel, nsel, ws, ws_bytes,
                           stream);
}

extern "C" int ann_select_lsh_buckets(const uint32_t *qbits, int n_q, const uint32_t *kbits, const int32_t *len, int H,
                                      int C, int n_bits, int band_bits, int radius, int BQ, int n_rep, int BK, int n_sel,
                                      int n_sink, int n_local, int32_t *sel, int32_t *nsel, void *ws, size_t ws_bytes,
                                      void *stream) {
    if (band_bits <= 0) return FASTAR_ERR_INVALID_ARG;
    return select_lsh_impl(qbits, n_q, kbits, len, H, C, n_bits, band_bits, radius, BQ, n_rep, BK, n_sel, n_sink, n_local,
                           sel, nsel, ws, ws_bytes, stream);
}
