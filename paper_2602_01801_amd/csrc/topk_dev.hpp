// Exact top-k of a row of integer scores by one workgroup: shared by the selection kernels.
#pragma once

#include <limits.h>

#include "common.hpp"

namespace fastar {

constexpr int TOPK_LDS_CAP = 8192; // row entries cached in LDS by the callers of topk_row
constexpr int TOPK_KPT = 16;       // rows of up to 256 * TOPK_KPT entries are selected from registers

// ---- exact top-k per row ----------------------------------------------------------------------------
// A row of n scores (row may point to global memory or to LDS).  The k = min(n_sel, n) largest are selected
// (ties: lowest index) and their indices written ascending to out[0..k), the rest of out[0..n_sel) padded with
// -1; *nsel_out = k.  Called by all 256 threads of a workgroup.
// keys: LDS staging for up to TOPK_LDS_CAP entries of a row in global memory, or nullptr (row read in place).
// k_cap: at most that many are selected (callers that admit only some entries as candidates pass their number; the
// others must score below every candidate).
// n_sink / n_local: the first / last entries of the row are forced (sink and local key blocks of AnnSA): they rank
// ahead of every real score, so they are always among the selected ones while n_sink + n_local <= n_sel.
__device__ __forceinline__ void topk_row(const int32_t *row, int n, int n_sel, int32_t *__restrict__ out,
                                         int32_t *__restrict__ nsel_out, unsigned *keys, int n_sink = 0, int n_local = 0,
                                         int k_cap = INT_MAX) {
    // Scores are sums of at most 64 products of 8-bit codes (or counts of equal hash bits): |score| < 2^21, and
    // anything below (the INT_MIN of a block without a live key) is clamped there, so an order-preserving key has
    // 22 bits: three passes over 8-bit digits (the first has 6 significant bits) select exactly.
    __shared__ unsigned hist[256];
    __shared__ unsigned sh_bin, sh_remaining;
    __shared__ unsigned wtot_a[4], wtot_b[4];
    const int tid = threadIdx.x;
    const int lane = lane_id(), wave = tid >> 6;
    const int k = min(min(n_sel, n), k_cap);
    if (tid == 0) *nsel_out = k;
    for (int t = k + tid; t < n_sel; t += 256) out[t] = -1;
    if (k == 0) return;
    if (k == n) {  // budget covers the row: everything, ascending
        for (int t = tid; t < n; t += 256) out[t] = t;
        return;
    }
    auto to_key0 = [](int32_t sc) -> unsigned { return (unsigned)(max(sc, -(1 << 21)) + (1 << 21)); };
    // key of entry t with score sc: real scores stay below 2^22, forced entries sit exactly there
    auto key_of = [&](int t, int32_t sc) -> unsigned {
        return (t < n_sink || t >= n - n_local) ? (1u << 22) : to_key0(sc);
    };
    if (n > 1024 && n <= TOPK_KPT * 256) {
        // Rows of 1025 to 4096 scores (shorter ones are done sooner by the three radix passes below, which take a
        // barrier per 256 entries in their compaction; longer ones do not fit the registers): each thread owns a run of consecutive entries and keeps
        // their keys in registers (key + 1, so that 0 stands for "no entry").  The k-th largest key is built bit by
        // bit (23 rounds of "how many keys reach this value": one compare per key, the wavefront's count through
        // scalar bit counts of the compare masks, one barrier per round), then one block scan of the per-thread
        // (greater, equal) counts places every selected index: 26 barriers in all, no atomics.
        const int kpt = (n + 255) / 256;
        unsigned my[TOPK_KPT];
        if (keys != nullptr) {   // row in global memory: coalesced loads, all in flight at once, staged through LDS
            int32_t v[TOPK_KPT];
#pragma unroll
            for (int e = 0; e < TOPK_KPT; ++e) {
                const int t = e * 256 + tid;
                v[e] = t < n ? row[t] : 0;
            }
#pragma unroll
            for (int e = 0; e < TOPK_KPT; ++e) {
                const int t = e * 256 + tid;
                if (t < n) keys[t] = key_of(t, v[e]);
            }
            __syncthreads();
#pragma unroll
            for (int e = 0; e < TOPK_KPT; ++e) {
                const int i = tid * kpt + e;
                my[e] = (e < kpt && i < n) ? keys[i] + 1u : 0u;
            }
        } else {
#pragma unroll
            for (int e = 0; e < TOPK_KPT; ++e) {
                const int i = tid * kpt + e;
                my[e] = (e < kpt && i < n) ? key_of(i, row[i]) + 1u : 0u;
            }
        }
        __shared__ unsigned cnt_w[2][4];
        auto count_ge = [&](unsigned cand, int buf) -> unsigned {   // entries with key + 1 >= cand, over the workgroup
            unsigned c = 0;
#pragma unroll
            for (int e = 0; e < TOPK_KPT; ++e) c += (unsigned)__popcll(__ballot(my[e] >= cand));
            if (lane == 0) cnt_w[buf][wave] = c;
            __syncthreads();
            return cnt_w[buf][0] + cnt_w[buf][1] + cnt_w[buf][2] + cnt_w[buf][3];
        };
        unsigned T = 0;
        int round = 0;
        for (int bit = 22; bit >= 0; --bit, ++round) {
            const unsigned cand = T | (1u << bit);
            if (count_ge(cand, round & 1) >= (unsigned)k) T = cand;
        }
        const unsigned need = (unsigned)k - count_ge(T + 1u, round & 1);   // ties at T that belong to the selection
        unsigned n_gt = 0, n_eq = 0;
#pragma unroll
        for (int e = 0; e < TOPK_KPT; ++e) {
            n_gt += my[e] > T ? 1u : 0u;
            n_eq += my[e] == T ? 1u : 0u;
        }
        const unsigned packed = (n_gt << 16) | n_eq;   // both totals stay below 4097
        unsigned incl = packed;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const unsigned o = __shfl_up(incl, off, WAVE);
            if (lane >= off) incl += o;
        }
        if (lane == 63) wtot_a[wave] = incl;
        __syncthreads();
        unsigned excl = incl - packed;
#pragma unroll
        for (int w = 0; w < 4; ++w)
            if (w < wave) excl += wtot_a[w];
        unsigned eq_rank = excl & 0xFFFFu;
        unsigned pos = (excl >> 16) + min(eq_rank, need);
#pragma unroll
        for (int e = 0; e < TOPK_KPT; ++e) {
            const bool take = my[e] > T || (my[e] == T && eq_rank < need);
            if (my[e] == T) eq_rank += 1;
            if (take) out[pos++] = tid * kpt + e;
        }
        return;
    }
    const bool cached = keys != nullptr && n <= TOPK_LDS_CAP;
    if (cached) {
        for (int t0 = 0; t0 < n; t0 += 4 * 256) {   // four loads in flight per thread
            int32_t v[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int t = t0 + e * 256 + tid;
                v[e] = t < n ? row[t] : 0;
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int t = t0 + e * 256 + tid;
                if (t < n) keys[t] = key_of(t, v[e]);
            }
        }
    }
    auto key_at = [&](int i) -> unsigned { return cached ? keys[i] : key_of(i, row[i]); };

    // radix select, most significant digit first: after the loop `prefix` is the k-th largest key and
    // `remaining` the number of entries equal to it that belong to the selection
    unsigned prefix = 0, mask = 0, remaining = (unsigned)k;
    for (int shift = 16; shift >= 0; shift -= 8) {
        hist[tid] = 0;
        __syncthreads();
        // The leading digits of a row's scores are often all alike: when every candidate of a wavefront falls into one
        // bin, one lane adds their number (64 additions to one LDS word are served one after the other).
        for (int base = 0; base < n; base += 256) {   // uniform trip count
            const int t = base + tid;
            unsigned bin = 0;
            bool act = false;
            if (t < n) {
                const unsigned u = key_at(t);
                act = (u & mask) == prefix;
                bin = (u >> shift) & 255u;
            }
            const unsigned long long m = __ballot(act);
            if (m) {
                const int first = __ffsll(m) - 1;
                const unsigned fbin = (unsigned)__shfl((int)bin, first, WAVE);
                if (__all(!act || bin == fbin)) {
                    if (lane == first) atomicAdd(&hist[fbin], (unsigned)__popcll(m));
                } else if (act) {
                    atomicAdd(&hist[bin], 1u);
                }
            }
        }
        __syncthreads();
        if (wave == 0) {
            // lane l owns bins 255-4l .. 252-4l (descending); find where the running count reaches `remaining`
            unsigned c[4], s = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                c[e] = hist[255 - 4 * lane - e];
                s += c[e];
            }
            unsigned incl = s;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                unsigned o = __shfl_up(incl, off, WAVE);
                if (lane >= off) incl += o;
            }
            unsigned before = incl - s;
            if (before < remaining && incl >= remaining) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (before < remaining && before + c[e] >= remaining) {
                        sh_bin = 255 - 4 * lane - e;
                        sh_remaining = remaining - before;
                        before = 0xFFFFFFFFu;  // stop
                    } else if (before != 0xFFFFFFFFu) {
                        before += c[e];
                    }
                }
            }
        }
        __syncthreads();
        prefix |= sh_bin << shift;
        mask |= 0xFFu << shift;
        remaining = sh_remaining;
    }
    const unsigned T = prefix, need = remaining;

    // ordered compaction
    unsigned eq_before = 0, out_before = 0;
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
    for (int base = 0; base < n; base += 256) {
        const int i = base + tid;
        const bool valid = i < n;
        const unsigned u = valid ? key_at(i) : 0u;
        const bool is_gt = valid && u > T, is_eq = valid && u == T;
        const unsigned long long m_eq = __ballot(is_eq);
        if (lane == 0) wtot_a[wave] = __popcll(m_eq);
        __syncthreads();
        unsigned eq_rank = eq_before + __popcll(m_eq & lt_mask), eq_total = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            if (w < wave) eq_rank += wtot_a[w];
            eq_total += wtot_a[w];
        }
        const bool take = is_gt || (is_eq && eq_rank < need);
        const unsigned long long m_take = __ballot(take);
        if (lane == 0) wtot_b[wave] = __popcll(m_take);
        __syncthreads();
        unsigned pos = out_before + __popcll(m_take & lt_mask), take_total = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            if (w < wave) pos += wtot_b[w];
            take_total += wtot_b[w];
        }
        if (take) out[pos] = i;
        eq_before += eq_total;
        out_before += take_total;
        __syncthreads();  // wtot_a / wtot_b are rewritten by the next chunk
    }
}

// Entries of a row that are candidates: score >= cand_min, or forced (first n_sink / last n_local).  All 256 threads.
__device__ __forceinline__ int count_candidates(const int32_t *row, int n, int n_sink, int n_local, int cand_min) {
    __shared__ int cand_w[4];
    int c = 0;
    for (int base = 0; base < n; base += 256) {   // uniform trip count
        const int t = base + threadIdx.x;
        const bool is_cand = t < n && (row[t] >= cand_min || t < n_sink || t >= n - n_local);
        c += __popcll(__ballot(is_cand));
    }
    if (lane_id() == 0) cand_w[threadIdx.x >> 6] = c;
    __syncthreads();
    return cand_w[0] + cand_w[1] + cand_w[2] + cand_w[3];
}

}  // namespace fastar
