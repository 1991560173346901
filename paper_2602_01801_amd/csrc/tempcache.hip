// TempCache (Sec. 5.2 of the paper, Lemma 1): merge one frame of new keys/values into the bounded
// per-head cache.  The steps, each a kernel on the caller's stream:
//   tc_match_window  (candidate list that fits LDS, probe = new key: the usual call) codes of the new keys AND the
//                 top-1 candidate slot of every token on exact integer code scores (int8 matrix cores), final in
//                 one launch; clears the group records of the matched slots
//   otherwise     encode (encode.hip) -> tc_match (candidate chunks over many workgroups, 64-bit atomicMax) ->
//                 tc_prep (unpack the match, clear the group records it will touch)
//   tc_verify     cosine test on the 8-bit quantised full-width keys as an int64 inequality; joiners
//                 register in their slot's group record (count, best joiner); age histogram of the live slots
//   tc_plan       per head: ranks of the unmerged tokens (ballot + prefix sum), evictions needed,
//                 victims = oldest untouched slots (histogram select over several workgroups, ordered compaction)
//   tc_apply      representative key, mean value, multiplicity, code, stamp of merged slots; appended
//                 tokens into victims / fresh slots; merge map
// All decisions are integer and order-independent (max / count), so the merge map is reproducible.
#include <limits.h>

#include <algorithm>

#include "encode_dev.hpp"

namespace fastar {

int encode_launch(const void *x, int dtype, int64_t n_vec, int d, const fastar_codec *codec, int r, int8_t *code,
                  unsigned long long *zero_fill, int64_t zero_n, hipStream_t s);

constexpr int SCORE_BIAS = 1 << 23;      // makes every score positive inside the packed arg-max key
constexpr int PLAN_SCRATCH_WORDS = 64 + 3 * 1024;  // per-head scratch of tc_plan_kernel (PS_STRIDE)
constexpr int HS_STRIDE = 8;             // per-head scalars: oldL, n_unmerged, e, n_victims, n_dropped, newL, 3 if the workspace is not clean, clean mark
constexpr int WS_CLEAN = 0x5A17C1EA;     // hs word 7 after a call: group records and plan scratch are all zero again
constexpr int WS_FAILED = 0x0BADC0DE;    // hs word 7 after a call whose plan gave up for the head: records and scratch are left as they are

typedef unsigned long long u64;

static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct CompressWs {
    size_t ck, cp, best, jstar, sbest, rank, victims, hs, ps, win, grp, total;
};
static CompressWs compress_ws(int H, int C, int n_new, int r) {
    CompressWs w;
    size_t o = 0;
    const size_t T = (size_t)H * (n_new > 0 ? n_new : 1);
    w.ck = o; o += align256(T * r);
    w.cp = o; o += align256(T * r);
    w.best = o; o += align256(T * 8);
    w.ps = o; o += align256((size_t)H * PLAN_SCRATCH_WORDS * 4);   // directly behind best: one zero fill covers both
    w.jstar = o; o += align256(T * 4);
    w.sbest = o; o += align256(T * 4);
    w.rank = o; o += align256(T * 4);
    w.victims = o; o += align256(T * 4);
    w.hs = o; o += align256((size_t)H * HS_STRIDE * 4);
    w.win = o; o += align256((size_t)H * C * 8);
    w.grp = o; o += align256((size_t)H * C * 4);
    w.total = o;
    return w;
}
size_t compress_ws_bytes(int H, int C, int n_new, int r) {
    if (H <= 0 || C <= 0 || n_new < 0 || r <= 0) return 0;
    return compress_ws(H, C, n_new, r).total;
}

// Running arg-max of one lane over the 16 scores a 32x32 matrix instruction leaves it (rows 8(v/4) + 4(lane/32) + v%4
// of a group of 32 candidates), with "earliest position" among equal scores at no extra cost: a score word carries
// its position among the 16 in its low four bits (one shift-add per score), so plain maxima pick (highest score, then
// earliest row), and a later group only replaces the best on a strictly higher score.  Callers present the
// candidates in ascending slot order without repeats, which makes this the smallest-slot rule of the match.
// Scores lie within +-2^21, missing candidates carry MATCH_NONE: both survive the shift by four.
constexpr int MATCH_NONE = -(1 << 26);       // score word of a missing candidate (minus its "penalty")
constexpr int MATCH_VALID = -(1 << 25);      // every real score is above, every missing one below
struct LaneBest {
    int s = INT_MIN, m = 0, g = 0;           // best score, its packed word, the group it came from
    __device__ __forceinline__ void take(const i32x16 &acc, int group) {
        int p[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) p[v] = (int)(((unsigned)acc[v] << 4) + (unsigned)(15 - v));
        int mx = p[0];
#pragma unroll
        for (int v = 1; v < 16; ++v) mx = max(mx, p[v]);
        const int sc = mx >> 4;
        if (sc > s) { s = sc; m = mx; g = group; }
    }
    // position of the best among the candidates (group * 32 + row), or -1 when no real candidate was seen
    __device__ __forceinline__ int pos(int g2) const {
        if (s <= MATCH_VALID) return -1;
        const int v = 15 - (m & 15);
        return g * 32 + 8 * (v >> 2) + 4 * g2 + (v & 3);
    }
    // (score, position) as one word ordered like the arg-max: higher score first, then the earlier position
    __device__ __forceinline__ u64 key(int g2, int pos0) const {
        const int p = pos(g2);
        return p < 0 ? 0ull : ((u64)(unsigned)(s + SCORE_BIAS) << 32) | (u64)(0xFFFFFFFFu - (unsigned)(pos0 + p));
    }
};

// ---- match -------------------------------------------------------------------------------------------
// D = A x B: A rows = 32 candidate slots (codes gathered by slot id), B columns = 32 tokens (probe codes).
// A lane therefore sees 16 candidates of one token per matrix instruction and keeps the best
// (score, lowest slot) as one 64-bit key: (score + bias) << 32 | ~slot.
// CAND_CHUNK = candidate positions scanned by one workgroup: 64 for a windowed candidate list (more, lighter
// workgroups hide the two dependent loads better), 256 for a scan of the whole cache (fewer atomics per token).
// Ties go to the smallest slot.  A scan of the whole cache (LIST false) visits the slots in ascending order, so the
// cheap "earliest position" arg-max of LaneBest is that rule.  A candidate list too long for the LDS window (LIST)
// comes in any order and may repeat ids: there every score is compared as the full (score, smallest slot) key.
template <int R, int CAND_CHUNK, bool LIST>
__global__ __launch_bounds__(256) void tc_match_kernel(const int8_t *__restrict__ code, const int32_t *__restrict__ len,
                                                       int C, const int8_t *__restrict__ cp, int n_new,
                                                       const int32_t *__restrict__ cand, int n_cand, int metric,
                                                       u64 *__restrict__ best) {
    constexpr int KS = R / 32;
    constexpr int NIT = CAND_CHUNK / 32;  // groups of 32 candidates per workgroup
    __shared__ __attribute__((aligned(16))) int cpen[4][CAND_CHUNK];   // minus the score penalty: -|code|^2 (metric 0), 0 (metric 1); MATCH_NONE: no candidate
    __shared__ __attribute__((aligned(16))) int cslotw[LIST ? 4 : 1][LIST ? CAND_CHUNK : 4];   // slot of every row (LIST)
    const int h = blockIdx.z;
    const int L = min(len[h], C);
    const int n_pos = LIST ? n_cand : L;
    const int pos0 = blockIdx.y * CAND_CHUNK;
    if (pos0 >= n_pos) return;  // uniform
    const int pos1 = min(pos0 + CAND_CHUNK, n_pos);
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int col = lane & 31, g2 = lane >> 5;
    const int tok = blockIdx.x * 128 + wave * 32 + col;
    const int8_t *cph = cp + (size_t)h * n_new * R;
    const int8_t *ch = code + (size_t)h * C * R;
    i32x4 bfrag[KS];
    {
        const int trow = min(tok, n_new - 1);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) bfrag[ks] = *(const i32x4 *)(cph + (size_t)trow * R + ks * 32 + 16 * g2);
    }
    // Two rounds of independent loads for the whole chunk (slot ids, then the codes they name) instead of
    // one dependent pair per group: the chunk costs two memory round trips, not 2 * NIT.
    int slot[NIT];
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int pos = pos0 + it * 32 + col;
        int sl = -1;
        if (pos < pos1) {
            sl = LIST ? cand[(size_t)h * n_cand + pos] : pos;
            if (sl < 0 || sl >= L) sl = -1;
        }
        slot[it] = sl;
    }
    i32x4 afrag[NIT][KS];
#pragma unroll
    for (int it = 0; it < NIT; ++it)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            i32x4 a = {0, 0, 0, 0};
            if (slot[it] >= 0) a = *(const i32x4 *)(ch + (size_t)slot[it] * R + ks * 32 + 16 * g2);
            afrag[it][ks] = a;
        }
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        int nn = 0;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int m = 0; m < 4; ++m) nn = dot4_i8((unsigned)afrag[it][ks][m], (unsigned)afrag[it][ks][m], nn);
        nn += shfl_xor(nn, 32);
        if (g2 == 0) {
            cpen[wave][it * 32 + col] = slot[it] >= 0 ? (metric == 0 ? -nn : 0) : MATCH_NONE;
            if (LIST) cslotw[wave][it * 32 + col] = slot[it];
        }
    }
    __syncthreads();  // every wavefront reads back only its own rows; the barrier orders write and read
    LaneBest lb;
    u64 mybest = 0;
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        if (pos0 + it * 32 >= pos1) break;  // uniform
        // the accumulator starts from minus the penalty of its rows and takes the product twice for 2 * dot:
        // the matrix unit does the arithmetic of the score
        i32x16 acc;
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            const i32x4 np = *(const i32x4 *)(&cpen[wave][it * 32 + 8 * q4 + 4 * g2]);
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[4 * q4 + e] = np[e];
        }
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) acc = mfma_i8_32x32x32(afrag[it][ks], bfrag[ks], acc);
        if (metric == 0) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) acc = mfma_i8_32x32x32(afrag[it][ks], bfrag[ks], acc);
        }
        if (LIST) {
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const i32x4 sl4 = *(const i32x4 *)(&cslotw[wave][it * 32 + 8 * q4 + 4 * g2]);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const u64 key = ((u64)(unsigned)(acc[4 * q4 + e] + SCORE_BIAS) << 32) | (u64)(0xFFFFFFFFu - (unsigned)sl4[e]);
                    if (sl4[e] >= 0 && key > mybest) mybest = key;
                }
            }
        } else {
            lb.take(acc, it);
        }
    }
    if (!LIST) mybest = lb.key(g2, pos0);   // position = slot
    {
        const unsigned lo = shfl_xor((unsigned)mybest, 32), hi = shfl_xor((unsigned)(mybest >> 32), 32);
        const u64 other = ((u64)hi << 32) | lo;
        if (other > mybest) mybest = other;
    }
    if (g2 == 0 && tok < n_new && mybest != 0) atomicMax(&best[(size_t)h * n_new + tok], mybest);
}

// ---- match against a candidate window held in LDS --------------------------------------------------------
// For a candidate list short enough to stage in LDS (the previous frame's slots: n_cand * (R + 8) bytes), one
// workgroup owns 64 tokens and sees every candidate, so the arg-max is final when it ends: no atomics, no packed
// keys to unpack, and the group records of the matched slots are cleared right here.  The eight wavefronts are
// (token half) x (quarter of the window): each takes every fourth step of 4 x 32 candidates, the partial arg-maxima
// meet through LDS.  The epilogue per 32 x 32 scores is plain integer ALU work, so two wavefronts per SIMD (not
// one) are what keeps the ALUs issuing.
// LDS: codes chunk-major ([16-byte chunk][candidate], conflict-free A-operand reads), slot ids, penalties.
// With ENC the kernel also is the call's encode step for its 64 tokens (probe = new key): it quantises and projects
// their rows while the window's loads are in flight, leaves the codes in ck for the apply step, and clears the
// eviction plan's scratch words (ps_all) for the launches behind it.
constexpr int WIN_THREADS = 512;
// What the fused tail of the window kernel needs from the verify step (defined further down).
template <bool BF16, int D>
struct VerifyRows;
constexpr int AGE_BINS = 1024;
template <int UN>
__device__ __forceinline__ void age_histogram_slice(const int32_t *__restrict__ len, const int32_t *__restrict__ stamp,
                                                    int C, int n_new, int frame_id, unsigned *__restrict__ ps,
                                                    int hist_word, int fut_word, unsigned *lhist);
struct VerifyArgs {   // the verify step's arguments, for the launch that runs it as its tail
    const void *K;
    int tau2_q16;
    uint8_t *merged;
    const int32_t *stamp;
    int frame_id, hist_word, fut_word;
};

// With VERIFY (workspaces that every call leaves clean, see tempcache_compress) the kernel is the verify step too: once
// the arg-max of its 64 tokens is final it runs the cosine test for them and registers the joiners; nothing is cleared
// here (records and plan scratch are clean on entry), and every workgroup adds its slice of the age histogram.
// TOKS: tokens per workgroup.  64 (two groups of 32 tokens, four wavefronts share each group's window scan) when the
// call is latency-bound; 256 (eight groups, one wavefront scans the whole window for its group) when there are many
// more workgroups than the chip holds at once: staging the window is then paid a quarter as often.
template <int R, bool ENC, bool BF16, int D, bool VERIFY, int TOKS>
__global__ __launch_bounds__(WIN_THREADS) void tc_match_window_kernel(const int8_t *__restrict__ code,
                                                              const int32_t *__restrict__ len, int C,
                                                              const int8_t *__restrict__ cp, int n_new,
                                                              const int32_t *__restrict__ cand, int n_cand, int metric,
                                                              int32_t *__restrict__ jstar, int32_t *__restrict__ sbest,
                                                              u64 *__restrict__ win, int32_t *__restrict__ grp,
                                                              const void *__restrict__ K_new,
                                                              const int8_t *__restrict__ Rm, float qscale, int shift,
                                                              int8_t *__restrict__ ck, unsigned *__restrict__ ps_all,
                                                              int ps_words, VerifyArgs va) {
    static_assert(!VERIFY || ENC, "the fused verify step reads the probe codes this kernel encoded");
    constexpr int KS = R / 32;
    constexpr int NCH = R / 16;  // 16-byte chunks per code
    extern __shared__ __attribute__((aligned(16))) unsigned char wlds[];
    const int n_pad = (n_cand + 31) & ~31;
    i32x4 *ccode = (i32x4 *)wlds;                       // [NCH][n_pad]
    int *cslot = (int *)(wlds + (size_t)NCH * n_pad * 16);  // [n_pad]
    int *cpen = cslot + n_pad;                          // [n_pad]
    constexpr int TG = TOKS / 32;                  // groups of 32 tokens
    constexpr int SPLIT = (WIN_THREADS / 64) / TG; // wavefronts sharing one group of 32 tokens, each on its share of the window
    static_assert(TG * SPLIT == WIN_THREADS / 64 && (TOKS == 64 || TOKS % 128 == 0), "token groups times window shares = wavefronts");
    __shared__ u64 partbest[SPLIT][TG][32];
    const int h = blockIdx.y;
    const int L = min(len[h], C);
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const int col = lane & 31, g2 = lane >> 5;
    const int tg = wave % TG, ch = wave / TG;
    const int8_t *ch_code = code + (size_t)h * C * R;
    // Tokens of this workgroup: [t0, t1).  64 tokens: its block.  256: an equal share of the frame (whole groups of 32
    // tokens), taken in blocks of 256 once the window is staged; the launcher sizes the grid so that no share is empty.
    const int per = TOKS < 256 ? TOKS : ((((n_new + (int)gridDim.x - 1) / (int)gridDim.x) + 31) & ~31);
    const int t0 = min((int)blockIdx.x * per, n_new), t1 = min(t0 + per, n_new);
    __shared__ __attribute__((aligned(16))) int8_t pcode[ENC ? TOKS * R : 16];
    i32x4 bfrag[KS];
    CodeMatrix<BF16, D, R> cm;
    // encoding: 16 tokens per wavefront and round; 64 tokens: wavefronts 0..3 once, 256 tokens: all eight twice
    constexpr int EROUNDS = TOKS >= 128 ? TOKS / 128 : 1;
    const bool enc_wave = ENC && (TOKS >= 128 || wave < 4);
    i32x4 xq[EROUNDS][D / 64];
    if (ENC && !VERIFY)
        for (int k = blockIdx.x * WIN_THREADS + tid; k < ps_words; k += gridDim.x * WIN_THREADS) ps_all[(size_t)h * ps_words + k] = 0u;
    if (enc_wave) cm.load(Rm, lane);
    // what a block of tokens needs before the window can be scanned for it: the rows to encode (ENC) or the probe
    // codes (B operand); for the workgroup's first block these loads are in flight while the window is staged
    auto load_block = [&](int base) {   // base: first token of the block
        if (enc_wave) {
#pragma unroll
            for (int er = 0; er < EROUNDS; ++er) {
                const int etok = base + 16 * (wave + 8 * er) + (lane & 15);  // token this lane helps to encode
                const char *row = (const char *)K_new + ((size_t)h * n_new + min(etok, n_new - 1)) * (size_t)D * (BF16 ? 2 : 4);
#pragma unroll
                for (int ks = 0; ks < D / 64; ++ks) xq[er][ks] = load_quantised<BF16>(row, ks, lane >> 4, qscale);
            }
        } else if (!ENC) {
            const int trow = min(base + tg * 32 + col, n_new - 1);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) bfrag[ks] = *(const i32x4 *)(cp + ((size_t)h * n_new + trow) * R + ks * 32 + 16 * g2);
        }
    };
    load_block(t0);
    // The candidate list is a SET of slots and ties go to the smallest slot, so the window is staged in ascending
    // slot order without repeats: position order then is slot order, which is all the arg-max below needs.
    //   1. every thread reads its entries of the list (ids outside [0, L) do not count) and whether the list already
    //      ascends (then it is staged as it stands: equal neighbours are the same slot and change nothing);
    //   2. otherwise the ids are sorted through a bitmap over the slot range they span, held where the codes will go
    //      (several passes when the range is wider than that area): set bits, count per wavefront, expand in order;
    //   3. the code rows of the sorted slots are gathered (one round of loads per batch, as before).
    constexpr int CPT = 8;          // list entries per thread: the window holds at most 148 KB / (R + 8) < 3840 ids
    constexpr int NOID = INT_MAX;   // key of an id that does not count
    __shared__ int s_flag, s_min, s_max, s_wtot[WIN_THREADS / 64];
    int ce[CPT];
    {
        bool descends = false;
        int vmin = NOID, vmax = -1;
        const int32_t *ch_cand = cand + (size_t)h * n_cand;
#pragma unroll
        for (int k = 0; k < CPT; ++k) {
            const int p = k * WIN_THREADS + tid;
            int v = NOID, before = -1;
            if (p < n_cand) {
                const int x = ch_cand[p];
                if (x >= 0 && x < L) v = x;
                if (p > 0) {
                    const int y = ch_cand[p - 1];
                    before = (y >= 0 && y < L) ? y : NOID;
                }
            }
            ce[k] = v;
            descends |= before > v;
            if (v != NOID) {
                vmin = min(vmin, v);
                vmax = max(vmax, v);
            }
        }
        if (tid == 0) {
            s_flag = 0;
            s_min = NOID;
            s_max = -1;
        }
        __syncthreads();
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            vmin = min(vmin, shfl_xor(vmin, off));
            vmax = max(vmax, shfl_xor(vmax, off));
        }
        const bool any_desc = __any(descends);
        if (lane == 0) {
            if (any_desc) atomicOr(&s_flag, 1);
            if (vmax >= 0) {
                atomicMin(&s_min, vmin);
                atomicMax(&s_max, vmax);
            }
        }
        __syncthreads();
    }
    int n_u;   // staged candidates (positions 0 .. n_u-1 of cslot; uniform over the workgroup)
    if (s_flag == 0) {
#pragma unroll
        for (int k = 0; k < CPT; ++k) {
            const int p = k * WIN_THREADS + tid;
            if (p < n_pad) cslot[p] = ce[k] == NOID ? -1 : ce[k];
        }
        n_u = n_cand;
        __syncthreads();
    } else {
        unsigned *bm = (unsigned *)wlds;                    // the code area: R * n_pad bytes
        const int bm_bits = 8 * R * n_pad;
        const int lo0 = s_min & ~31, hi = s_max + 1;
        int base = 0;
        for (int lo = lo0; lo < hi; lo += bm_bits) {       // uniform
            const int nbits = min(hi - lo, bm_bits);
            const int nw = (nbits + 31) >> 5;
            for (int w = tid; w < nw; w += WIN_THREADS) bm[w] = 0u;
            __syncthreads();
#pragma unroll
            for (int k = 0; k < CPT; ++k) {
                const int v = ce[k];
                if (v != NOID && v >= lo && v - lo < nbits) atomicOr(&bm[(v - lo) >> 5], 1u << ((v - lo) & 31));
            }
            __syncthreads();
            // a wavefront owns a contiguous run of words, its lanes take them 64 at a time
            const int wpw = (nw + WIN_THREADS / 64 - 1) / (WIN_THREADS / 64);
            const int w0 = min(wave * wpw, nw), w1 = min(w0 + wpw, nw);
            int c = 0;
            for (int w = w0 + lane; w < w1; w += 64) c += __popc(bm[w]);
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) c += shfl_xor(c, off);
            if (lane == 0) s_wtot[wave] = c;
            __syncthreads();
            int pos = base, tot = 0;
#pragma unroll
            for (int ww = 0; ww < WIN_THREADS / 64; ++ww) {
                const int t = s_wtot[ww];
                if (ww < wave) pos += t;
                tot += t;
            }
            for (int wb = w0; wb < w1; wb += 64) {         // uniform over the wavefront
                const int w = wb + lane;
                unsigned bits = w < w1 ? bm[w] : 0u;
                const int mine = __popc(bits);
                int incl = mine;
#pragma unroll
                for (int off = 1; off < 64; off <<= 1) {
                    const int o = __shfl_up(incl, off, WAVE);
                    if (lane >= off) incl += o;
                }
                int q = pos + incl - mine;
                while (bits) {
                    cslot[q++] = lo + 32 * w + (__ffs(bits) - 1);
                    bits &= bits - 1;
                }
                pos += __shfl(incl, 63, WAVE);
            }
            base += tot;
            __syncthreads();   // the bitmap may be cleared again; cslot is complete after the last pass
        }
        n_u = base;
    }
    const int n_stage = (n_u + 31) & ~31;   // <= n_pad
    // Code rows in batches of independent loads, so a batch costs one memory round trip however many rows it holds.
    constexpr int BATCH = 128 / R;  // candidates per thread and batch (32 code registers)
    for (int p0 = 0; p0 < n_stage; p0 += WIN_THREADS * BATCH) {
        int sl[BATCH];
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const int p = p0 + u * WIN_THREADS + tid;
            sl[u] = p < n_u ? cslot[p] : -1;
        }
        i32x4 row[BATCH][NCH];
#pragma unroll
        for (int u = 0; u < BATCH; ++u)
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                i32x4 v = {0, 0, 0, 0};
                if (sl[u] >= 0) v = *(const i32x4 *)(ch_code + (size_t)sl[u] * R + c * 16);
                row[u][c] = v;
            }
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const int p = p0 + u * WIN_THREADS + tid;
            if (p < n_stage) {
                int nn = 0;
#pragma unroll
                for (int c = 0; c < NCH; ++c) {
                    ccode[c * n_pad + p] = row[u][c];
#pragma unroll
                    for (int m = 0; m < 4; ++m) nn = dot4_i8((unsigned)row[u][c][m], (unsigned)row[u][c][m], nn);
                }
                if (p >= n_u) cslot[p] = -1;
                cpen[p] = sl[u] >= 0 ? (metric == 0 ? -nn : 0) : MATCH_NONE;  // minus the penalty
            }
        }
    }
    __shared__ int vj[TOKS], vs[TOKS];
    for (int base = t0; base < t1; base += TOKS) {
    const int lim = min(base + TOKS, t1);   // this block's tokens: [base, lim)
    const int tok = base + tg * 32 + col;
    if (base != t0) {
        __syncthreads();   // the previous block's probe codes and arg-maxima have been read
        load_block(base);
    }
    if (enc_wave) {
#pragma unroll
        for (int er = 0; er < EROUNDS; ++er) {
            const int etok = base + 16 * (wave + 8 * er) + (lane & 15);
#pragma unroll
            for (int cb = 0; cb < R / 16; ++cb) {
                const unsigned w = cm.code_word(xq[er], cb, shift);
                *(unsigned *)(pcode + (16 * (wave + 8 * er) + (lane & 15)) * R + cb * 16 + 4 * (lane >> 4)) = w;
                if (etok < lim) *(unsigned *)(ck + ((size_t)h * n_new + etok) * R + cb * 16 + 4 * (lane >> 4)) = w;
            }
        }
    }
    __syncthreads();
    if (ENC) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) bfrag[ks] = *(const i32x4 *)(pcode + (tg * 32 + col) * R + ks * 32 + 16 * g2);
    }
    // Running arg-max of a lane over the 16 scores per group its accumulators hold: only the best score and the group
    // it came from are kept in the loop (a maximum tree and one compare-select per group; a later group replaces the
    // best only on a strictly higher score, so the earliest group wins among equals); which of the group's rows it was
    // is looked up once, after the loop, by recomputing that group's 16 scores for this lane's token.
    int bs = INT_MIN, bg = 0;
    // a wavefront whose 32 tokens all lie beyond the block's end scans nothing (uniform over the wavefront)
    const int n_groups = base + tg * 32 < lim ? n_stage / 32 : 0;
    // squared distance: 2 * dot, the product is accumulated twice; inner product: the second product is with zero
    i32x4 bfrag2[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int e = 0; e < 4; ++e) bfrag2[ks][e] = metric == 0 ? bfrag[ks][e] : 0;
    if constexpr (TOKS >= 256) {
        // Long scans (one wavefront, the whole window): two groups of 32 candidates per step in three rotating operand
        // sets, so that the reads of step t + 2, the matrix instructions of step t + 1 and the maxima of step t are in
        // flight together (a wavefront issues in order: without the rotation its matrix and vector phases alternate).
        // Steps past the end repeat the last group, which changes nothing: only a strictly higher score replaces the best.
        constexpr int UNR = 2;
        struct ScanSet {
            i32x4 a[UNR][KS];
            i32x16 acc[UNR];
        };
        const int n_it = n_groups > ch * UNR ? (n_groups - ch * UNR + SPLIT * UNR - 1) / (SPLIT * UNR) : 0;
        auto group_of = [&](int it, int u) { return min((ch + it * SPLIT) * UNR + u, n_groups - 1); };
        auto rd = [&](ScanSet &s, int it) {
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                const int gi = group_of(it, u);
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) s.a[u][ks] = ccode[(2 * ks + g2) * n_pad + gi * 32 + col];
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {   // minus the penalty of the accumulator's rows
                    const i32x4 np = *(const i32x4 *)(&cpen[gi * 32 + 8 * q4 + 4 * g2]);
#pragma unroll
                    for (int e = 0; e < 4; ++e) s.acc[u][4 * q4 + e] = np[e];
                }
            }
        };
        auto mm = [&](ScanSet &s) {
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) s.acc[u] = mfma_i8_32x32x32(s.a[u][ks], bfrag[ks], s.acc[u]);
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) s.acc[u] = mfma_i8_32x32x32(s.a[u][ks], bfrag2[ks], s.acc[u]);
            }
        };
        auto red = [&](const ScanSet &s, int it) {
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                int mx = s.acc[u][0];
#pragma unroll
                for (int v = 1; v < 16; ++v) mx = max(mx, s.acc[u][v]);
                const bool better = mx > bs;
                bs = better ? mx : bs;
                bg = better ? group_of(it, u) : bg;
            }
        };
        if (n_it > 0) {
            ScanSet s0, s1, s2;
            rd(s0, 0);
            rd(s1, 1);
            mm(s0);
            for (int it = 0; it < n_it; it += 3) {
                rd(s2, it + 2);
                mm(s1);
                red(s0, it);
                rd(s0, it + 3);
                mm(s2);
                red(s1, it + 1);
                rd(s1, it + 4);
                mm(s0);
                red(s2, it + 2);
            }
        }
    } else {
    // Four groups of 32 candidates per step, their operand reads and matrix instructions issued together
    // (a group repeated at the ragged end changes nothing: only a strictly higher score replaces the best).
    constexpr int UNR = 4;
    for (int g0 = ch * UNR; g0 < n_groups; g0 += SPLIT * UNR) {
        i32x4 afrag[UNR][KS];
        i32x16 acc[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int gi = min(g0 + u, n_groups - 1);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) afrag[u][ks] = ccode[(2 * ks + g2) * n_pad + gi * 32 + col];
            // the accumulator starts from minus the penalty of its rows: the matrix unit does the subtraction
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const i32x4 np = *(const i32x4 *)(&cpen[gi * 32 + 8 * q4 + 4 * g2]);
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[u][4 * q4 + e] = np[e];
            }
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) acc[u] = mfma_i8_32x32x32(afrag[u][ks], bfrag[ks], acc[u]);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) acc[u] = mfma_i8_32x32x32(afrag[u][ks], bfrag2[ks], acc[u]);
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            int mx = acc[u][0];
#pragma unroll
            for (int v = 1; v < 16; ++v) mx = max(mx, acc[u][v]);
            const bool better = mx > bs;
            bs = better ? mx : bs;
            bg = better ? min(g0 + u, n_groups - 1) : bg;
        }
    }
    }
    u64 mybest = 0;
    if (bs > MATCH_VALID) {   // some real candidate was seen: the earliest row of group bg that reaches the best score
        i32x4 pc[NCH];
        const int8_t *prow = ENC ? pcode + (tg * 32 + col) * R : cp + ((size_t)h * n_new + min(tok, n_new - 1)) * R;
#pragma unroll
        for (int c = 0; c < NCH; ++c) pc[c] = *(const i32x4 *)(prow + 16 * c);
        int pos = -1;
#pragma unroll
        for (int v = 15; v >= 0; --v) {
            const int row = bg * 32 + 8 * (v >> 2) + 4 * g2 + (v & 3);
            int dot = 0;
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                const i32x4 cc = ccode[c * n_pad + row];
#pragma unroll
                for (int m = 0; m < 4; ++m) dot = dot4_i8((unsigned)cc[m], (unsigned)pc[c][m], dot);
            }
            const int S = (metric == 0 ? 2 * dot : dot) + cpen[row];
            pos = S == bs ? row : pos;
        }
        if (pos >= 0) mybest = ((u64)(unsigned)(bs + SCORE_BIAS) << 32) | (u64)(0xFFFFFFFFu - (unsigned)pos);
    }
    {
        const unsigned lo = shfl_xor((unsigned)mybest, 32), hi = shfl_xor((unsigned)(mybest >> 32), 32);
        const u64 other = ((u64)hi << 32) | lo;
        if (other > mybest) mybest = other;
    }
    if (g2 == 0) partbest[ch][tg][col] = mybest;
    __syncthreads();
    if (ch == 0 && g2 == 0) {
        int j = -1, S = 0;
        if (tok < lim) {
#pragma unroll
            for (int c = 1; c < SPLIT; ++c) {
                const u64 other = partbest[c][tg][col];
                if (other > mybest) mybest = other;
            }
            if (mybest != 0) {
                j = cslot[(int)(0xFFFFFFFFu - (unsigned)mybest)];   // position in the window -> slot
                S = (int)(unsigned)(mybest >> 32) - SCORE_BIAS;
                if (!VERIFY) {
                    win[(size_t)h * C + j] = 0;
                    grp[(size_t)h * C + j] = 0;
                }
            }
            jstar[(size_t)h * n_new + tok] = j;
            sbest[(size_t)h * n_new + tok] = S;
        }
        if (VERIFY) {
            vj[tg * 32 + col] = j;
            vs[tg * 32 + col] = S;
        }
    }
    if constexpr (VERIFY) {
        __syncthreads();
        constexpr int NPASS = TOKS * 16 / WIN_THREADS;   // tokens per 16-lane group
        constexpr int PB = TOKS >= 256 ? 8 : 2;          // passes whose rows are loaded together (registers)
#pragma unroll
        for (int p0 = 0; p0 < NPASS; p0 += PB) {
            VerifyRows<BF16, D> vr[PB];
#pragma unroll
            for (int pass = 0; pass < PB; ++pass) {   // every row this group will need, in one round of loads
                const int t = (p0 + pass) * (WIN_THREADS / 16) + (tid >> 4);
                const int i = min(base + t, n_new - 1);
                vr[pass].load(va.K, K_new, pcode + t * R, R, C, n_new, metric, h, i, tid & 15, vj[t]);
            }
#pragma unroll
            for (int pass = 0; pass < PB; ++pass) {
                const int t = (p0 + pass) * (WIN_THREADS / 16) + (tid >> 4);
                const int i = base + t;
                if (i < lim)   // whole 16-lane groups
                    vr[pass].decide(C, n_new, qscale, metric, va.tau2_q16, win, grp, va.merged, h, i, tid & 15, vj[t], vs[t]);
            }
        }
    }
    if constexpr (TOKS < 256) break;   // one block per workgroup: the grid covers the tokens (and the compiler sees no loop)
    }   // blocks of tokens
    if constexpr (VERIFY) {
        __shared__ unsigned lhist[AGE_BINS];
        __syncthreads();
        age_histogram_slice<(TOKS >= 256 ? 20 : 4)>(len, va.stamp, C, n_new, va.frame_id, ps_all + (size_t)h * ps_words,
                                                    va.hist_word, va.fut_word, lhist);
    }
}
static size_t match_window_lds(int n_cand, int r) { return (size_t)((n_cand + 31) & ~31) * (size_t)(r + 8); }
// dynamic LDS of the window kernel; with the static arrays of its largest instantiation (r = 64, fused verify: 10.6 KB)
// it stays within the 160 KB of a compute unit
constexpr size_t WINDOW_LDS_MAX = 148 * 1024;
// static LDS of the wide (256 tokens per workgroup) instantiations: probe codes, verify hand-over, partial results,
// age histogram, a few words; what is left of a compute unit's 160 KB is their window
static constexpr size_t wide_window_lds_max(int r) { return (size_t)160 * 1024 - ((size_t)256 * r + 256 * 8 + 2048 + 4096 + 256); }
template <int R, bool ENC, bool BF16, int D, bool VERIFY, int TOKS>
static int allow_window_lds() {
    const size_t lim = TOKS == 64 ? WINDOW_LDS_MAX : wide_window_lds_max(R);
    return hipFuncSetAttribute((const void *)tc_match_window_kernel<R, ENC, BF16, D, VERIFY, TOKS>,
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lim) == hipSuccess
               ? FASTAR_OK
               : FASTAR_ERR_HIP;
}
struct PlanResidency;
static int plan_residency(PlanResidency *out);
static int plan_residency_setup();
// every instantiation of the window kernel may use more than the default 64 KB of dynamic LDS: requested once per device
int tempcache_setup() {
    if (const int rc = plan_residency_setup(); rc != FASTAR_OK) return rc;
    static DeviceOnce once;
    return once.run([](int) {
        int rc = FASTAR_OK;
#define FASTAR_ALLOW(RR, BF, DD)                                                       \
    do {                                                                               \
        if (rc == FASTAR_OK) rc = allow_window_lds<RR, true, BF, DD, true, 64>();      \
        if (rc == FASTAR_OK) rc = allow_window_lds<RR, true, BF, DD, false, 64>();     \
        if (rc == FASTAR_OK) rc = allow_window_lds<RR, true, BF, DD, true, 256>();     \
        if (rc == FASTAR_OK) rc = allow_window_lds<RR, true, BF, DD, false, 256>();    \
    } while (0)
        FASTAR_ALLOW(32, true, 128); FASTAR_ALLOW(32, false, 128); FASTAR_ALLOW(32, true, 64); FASTAR_ALLOW(32, false, 64);
        FASTAR_ALLOW(64, true, 128); FASTAR_ALLOW(64, false, 128); FASTAR_ALLOW(64, true, 64); FASTAR_ALLOW(64, false, 64);
#undef FASTAR_ALLOW
        if (rc == FASTAR_OK) rc = allow_window_lds<32, false, true, 128, false, 64>();
        if (rc == FASTAR_OK) rc = allow_window_lds<64, false, true, 128, false, 64>();
        return rc;
    });
}
template <int R, bool ENC, bool BF16, int D, bool VERIFY, int TOKS, typename... Args>
static int launch_match_window(dim3 grid, size_t lds, hipStream_t s, Args... args) {
    hipLaunchKernelGGL((tc_match_window_kernel<R, ENC, BF16, D, VERIFY, TOKS>), grid, dim3(WIN_THREADS), lds, s, args...);
    FASTAR_LAUNCH_CHECK();
    return FASTAR_OK;
}

// ---- prep (only behind the chunked match, which leaves packed arg-max keys) ---------------------------------
// Unpacks the match and clears the per-slot group records it will touch.
__global__ __launch_bounds__(256) void tc_prep_kernel(const u64 *__restrict__ best, int n_new, int C,
                                                      const int32_t *__restrict__ cand, int n_cand,
                                                      int32_t *__restrict__ jstar, int32_t *__restrict__ sbest,
                                                      u64 *__restrict__ win, int32_t *__restrict__ grp) {
    const int h = blockIdx.y;
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_new) return;
    const u64 key = best[(size_t)h * n_new + i];
    int j = -1, S = 0;
    if (key != 0) {
        j = (int)(0xFFFFFFFFu - (unsigned)key);   // the low word counts down with the slot: ties went to the smallest
        S = (int)(unsigned)(key >> 32) - SCORE_BIAS;
        win[(size_t)h * C + j] = 0;
        grp[(size_t)h * C + j] = 0;
    }
    jstar[(size_t)h * n_new + i] = j;
    sbest[(size_t)h * n_new + i] = S;
}

// Per head, a histogram of the live slots' ages (frame_id - stamp, 1024 bins, the last one collecting everything
// older) for the eviction plan: the verify launch, a whole grid, reads the stamps, where the plan has few
// workgroups per head.  Every workgroup of the launch adds its slice of the slots.  Called by whole workgroups.
// UN: 16-byte loads per lane in flight before the first is used (a slice read in one round trip when it fits).
template <int UN>
__device__ __forceinline__ void age_histogram_slice(const int32_t *__restrict__ len, const int32_t *__restrict__ stamp,
                                                    int C, int n_new, int frame_id, unsigned *__restrict__ ps,
                                                    int hist_word, int fut_word, unsigned *lhist) {
    const int h = blockIdx.y;
    const int L = min(len[h], C);
    if (hist_word < 0) return;   // uniform over the launch: the plan counts the ages itself
    if (L + n_new <= C) return;  // uniform over the head: no eviction can be needed
    for (int k = threadIdx.x; k < AGE_BINS; k += blockDim.x) lhist[k] = 0;
    __syncthreads();
    // every workgroup takes a run of slots that starts on a multiple of four, four consecutive stamps per lane and load
    // (16 bytes when the head's row is aligned), four such loads in flight before the first is used
    const int chunk = ((L + gridDim.x - 1) / gridDim.x + 3) & ~3;
    const int j0 = min((int)blockIdx.x * chunk, L), j1 = min(j0 + chunk, L);
    const int32_t *st = stamp + (size_t)h * C;
    const bool vec = (((uintptr_t)st) & 15) == 0;
    bool future = false;
    // Neighbouring slots were mostly written by the same frame: when all of a wavefront's slots fall into one bin, one
    // lane adds their number (hundreds of additions to one LDS word would be served one after the other).
    for (int jb = j0; jb < j1; jb += (int)blockDim.x * 4 * UN) {   // uniform trip count
        int sv[UN][4];
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int j = jb + (u * (int)blockDim.x + (int)threadIdx.x) * 4;
            if (vec && j + 3 < j1) {
                const i32x4 v = *(const i32x4 *)(st + j);
                sv[u][0] = v[0]; sv[u][1] = v[1]; sv[u][2] = v[2]; sv[u][3] = v[3];
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) sv[u][e] = j + e < j1 ? st[j + e] : 0;
            }
        }
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int j = jb + (u * (int)blockDim.x + (int)threadIdx.x) * 4;
            unsigned bin[4];
            int n_act = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const bool act = j + e < j1;
                if (act && sv[u][e] > frame_id) future = true;
                bin[e] = min((unsigned)frame_id - (unsigned)sv[u][e], (unsigned)(AGE_BINS - 1));
                n_act += act ? 1 : 0;
            }
            const u64 m = __ballot(n_act > 0);
            if (m) {   // uniform
                const int first = __ffsll((unsigned long long)m) - 1;
                const unsigned fbin = (unsigned)__shfl((int)bin[0], first);   // an active lane's first slot is active
                bool same = true;
#pragma unroll
                for (int e = 0; e < 4; ++e) same = same && (j + e >= j1 || bin[e] == fbin);
                if (__all(same)) {
                    int tot = n_act;
#pragma unroll
                    for (int off = 32; off >= 1; off >>= 1) tot += shfl_xor(tot, off);
                    if (lane_id() == first) atomicAdd(&lhist[fbin], (unsigned)tot);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (j + e < j1) atomicAdd(&lhist[bin[e]], 1u);
                }
            }
        }
    }
    __syncthreads();
    for (int k = threadIdx.x; k < AGE_BINS; k += blockDim.x)
        if (lhist[k]) atomicAdd(&ps[hist_word + k], lhist[k]);
    if (__any(future) && lane_id() == 0) atomicOr(&ps[fut_word], 1u);
}

// ---- row pieces: 16 lanes share one row of D elements ----------------------------------------------------
template <bool BF16, int D>
struct RowPiece {
    static constexpr int EPL = D / 16;  // elements per lane
    __device__ static __forceinline__ void load(const void *base, size_t row, int l16, float *out) {
        if (BF16) {
            const unsigned short *p = (const unsigned short *)base + row * D + l16 * EPL;
            if (EPL == 8) {
                u32x4 w = *(const u32x4 *)p;
#pragma unroll
                for (int e = 0; e < 4; ++e) { out[2 * e] = bf16_lo(w[e]); out[2 * e + 1] = bf16_hi(w[e]); }
            } else {
                u32x2 w = *(const u32x2 *)p;
#pragma unroll
                for (int e = 0; e < 2; ++e) { out[2 * e] = bf16_lo(w[e]); out[2 * e + 1] = bf16_hi(w[e]); }
            }
        } else {
            const float *p = (const float *)base + row * D + l16 * EPL;
#pragma unroll
            for (int e = 0; e < EPL; e += 4) {
                f32x4 w = *(const f32x4 *)(p + e);
                out[e] = w[0]; out[e + 1] = w[1]; out[e + 2] = w[2]; out[e + 3] = w[3];
            }
        }
    }
    __device__ static __forceinline__ void store(void *base, size_t row, int l16, const float *v) {
        if (BF16) {
            unsigned short *p = (unsigned short *)base + row * D + l16 * EPL;
            if (EPL == 8) {
                u32x4 w;
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = pack_bf16x2(v[2 * e], v[2 * e + 1]);
                *(u32x4 *)p = w;
            } else {
                u32x2 w;
#pragma unroll
                for (int e = 0; e < 2; ++e) w[e] = pack_bf16x2(v[2 * e], v[2 * e + 1]);
                *(u32x2 *)p = w;
            }
        } else {
            float *p = (float *)base + row * D + l16 * EPL;
#pragma unroll
            for (int e = 0; e < EPL; e += 4) {
                f32x4 w = {v[e], v[e + 1], v[e + 2], v[e + 3]};
                *(f32x4 *)(p + e) = w;
            }
        }
    }
    // this lane's piece of a row as raw bits (held in registers between an early load and a late store)
    struct Raw {
        u32x4 w[(EPL * (BF16 ? 2 : 4) + 15) / 16];
    };
    __device__ static __forceinline__ Raw load_raw(const void *base, size_t row, int l16) {
        constexpr int BYTES = EPL * (BF16 ? 2 : 4);
        const char *s = (const char *)base + (row * D + (size_t)l16 * EPL) * (BF16 ? 2 : 4);
        Raw r;
        if (BYTES == 8) {
            const u32x2 v = *(const u32x2 *)s;
            r.w[0][0] = v[0]; r.w[0][1] = v[1]; r.w[0][2] = 0; r.w[0][3] = 0;
        } else {
#pragma unroll
            for (int b = 0; b < BYTES; b += 16) r.w[b / 16] = *(const u32x4 *)(s + b);
        }
        return r;
    }
    __device__ static __forceinline__ void store_raw(void *base, size_t row, int l16, const Raw &r) {
        constexpr int BYTES = EPL * (BF16 ? 2 : 4);
        char *d = (char *)base + (row * D + (size_t)l16 * EPL) * (BF16 ? 2 : 4);
        if (BYTES == 8) {
            u32x2 v = {r.w[0][0], r.w[0][1]};
            *(u32x2 *)d = v;
        } else {
#pragma unroll
            for (int b = 0; b < BYTES; b += 16) *(u32x4 *)(d + b) = r.w[b / 16];
        }
    }
    // raw bits -> float values of the piece
    __device__ static __forceinline__ void unpack(const Raw &r, float *out) {
        if (BF16) {
#pragma unroll
            for (int e = 0; e < EPL / 2; ++e) {
                const unsigned w = r.w[e / 4][e % 4];
                out[2 * e] = bf16_lo(w);
                out[2 * e + 1] = bf16_hi(w);
            }
        } else {
#pragma unroll
            for (int e = 0; e < EPL; ++e) out[e] = __uint_as_float(r.w[e / 4][e % 4]);
        }
    }
    // bit copy of this lane's piece of a row
    __device__ static __forceinline__ void copy(void *dst, size_t drow, const void *src, size_t srow, int l16) {
        constexpr int BYTES = EPL * (BF16 ? 2 : 4);
        const char *s = (const char *)src + (srow * D + (size_t)l16 * EPL) * (BF16 ? 2 : 4);
        char *d = (char *)dst + (drow * D + (size_t)l16 * EPL) * (BF16 ? 2 : 4);
        if (BYTES == 8) {
            *(u32x2 *)d = *(const u32x2 *)s;
        } else {
#pragma unroll
            for (int b = 0; b < BYTES; b += 16) *(u32x4 *)(d + b) = *(const u32x4 *)(s + b);
        }
    }
};

__device__ __forceinline__ int group16_sum(int v) {
    v += shfl_xor(v, 1);
    v += shfl_xor(v, 2);
    v += shfl_xor(v, 4);
    v += shfl_xor(v, 8);
    return v;
}

// ---- verify --------------------------------------------------------------------------------------------
template <bool BF16, int D>
__device__ __forceinline__ void verify_token(const void *__restrict__ K, const void *__restrict__ K_new,
                                             const int8_t *__restrict__ cp, int r, int C, int n_new, float qscale,
                                             int metric, int tau2_q16, const int32_t *__restrict__ jstar,
                                             const int32_t *__restrict__ sbest, u64 *__restrict__ win,
                                             int32_t *__restrict__ grp, uint8_t *__restrict__ merged, int h, int i,
                                             int l16);

template <bool BF16, int D>
__global__ __launch_bounds__(256) void tc_verify_kernel(const void *__restrict__ K, const void *__restrict__ K_new,
                                                        const int8_t *__restrict__ cp, int r, int C, int n_new,
                                                        float qscale, int metric, int tau2_q16,
                                                        const int32_t *__restrict__ jstar,
                                                        const int32_t *__restrict__ sbest, u64 *__restrict__ win,
                                                        int32_t *__restrict__ grp, uint8_t *__restrict__ merged,
                                                        const int32_t *__restrict__ len,
                                                        const int32_t *__restrict__ stamp, int frame_id,
                                                        unsigned *__restrict__ plan_scratch, int hist_word,
                                                        int fut_word, int scratch_words) {
    typedef RowPiece<BF16, D> RP;
    __shared__ unsigned lhist[AGE_BINS];
    const int h = blockIdx.y;
    const int l16 = threadIdx.x & 15;
    const int i = blockIdx.x * (blockDim.x / 16) + (threadIdx.x >> 4);
    if (i < n_new) verify_token<BF16, D>(K, K_new, cp, r, C, n_new, qscale, metric, tau2_q16, jstar, sbest, win, grp,
                                         merged, h, i, l16);  // whole 16-lane groups
    age_histogram_slice<4>(len, stamp, C, n_new, frame_id, plan_scratch + (size_t)h * scratch_words, hist_word, fut_word,
                        lhist);
}

// Token i of head h, matched to slot j with code score W (j < 0: no candidate); cprow = the token's probe code.
// Two halves, so that a caller with several tokens per lane group can issue all their loads first.  Whole 16-lane groups.
template <bool BF16, int D>
struct VerifyRows {
    typename RowPiece<BF16, D>::Raw ra, rb;   // raw bits: half the registers of the float values while the loads are in flight
    unsigned cw;
    __device__ __forceinline__ void load(const void *__restrict__ K, const void *__restrict__ K_new, const int8_t *cprow,
                                         int r, int C, int n_new, int metric, int h, int i, int l16, int j) {
        typedef RowPiece<BF16, D> RP;
        ra = RP::load_raw(K_new, (size_t)h * n_new + i, l16);
        cw = (metric == 0 && l16 < r / 4) ? ((const unsigned *)cprow)[l16] : 0u;
        if (j >= 0) rb = RP::load_raw(K, (size_t)h * C + j, l16);
    }
    __device__ __forceinline__ void decide(int C, int n_new, float qscale, int metric, int tau2_q16, u64 *__restrict__ win,
                                           int32_t *__restrict__ grp, uint8_t *__restrict__ merged, int h, int i,
                                           int l16, int j, int W) const {
        typedef RowPiece<BF16, D> RP;
        const int nn = group16_sum(dot4_i8(cw, cw, 0));  // |probe code|^2 (r <= 64: at most 16 words)
        bool is_merged = false;
        if (j >= 0) {
            float a[RP::EPL], b[RP::EPL];
            RP::unpack(ra, a);
            RP::unpack(rb, b);
            int dot = 0, na = 0, nb = 0;
#pragma unroll
            for (int e = 0; e < RP::EPL; ++e) {
                const int qa = quant8(a[e], qscale), qb = quant8(b[e], qscale);
                dot += qa * qb;
                na += qa * qa;
                nb += qb * qb;
            }
            dot = group16_sum(dot);
            na = group16_sum(na);
            nb = group16_sum(nb);
            is_merged = dot > 0 && (long long)dot * dot * 65536ll >= (long long)tau2_q16 * na * nb;
            if (is_merged && l16 == 0) {
                if (metric == 0) W -= nn;
                const u64 key = ((u64)(unsigned)(W + SCORE_BIAS) << 32) | (u64)(0xFFFFFFFFu - (unsigned)i);
                atomicMax(&win[(size_t)h * C + j], key);
                atomicAdd(&grp[(size_t)h * C + j], 1);
            }
        }
        if (l16 == 0) merged[(size_t)h * n_new + i] = is_merged ? 1 : 0;
    }
};
template <bool BF16, int D>
__device__ __forceinline__ void verify_core(const void *__restrict__ K, const void *__restrict__ K_new,
                                            const int8_t *cprow, int r, int C, int n_new, float qscale, int metric,
                                            int tau2_q16, u64 *__restrict__ win, int32_t *__restrict__ grp,
                                            uint8_t *__restrict__ merged, int h, int i, int l16, int j, int W) {
    VerifyRows<BF16, D> v;
    v.load(K, K_new, cprow, r, C, n_new, metric, h, i, l16, j);
    v.decide(C, n_new, qscale, metric, tau2_q16, win, grp, merged, h, i, l16, j, W);
}

template <bool BF16, int D>
__device__ __forceinline__ void verify_token(const void *__restrict__ K, const void *__restrict__ K_new,
                                             const int8_t *__restrict__ cp, int r, int C, int n_new, float qscale,
                                             int metric, int tau2_q16, const int32_t *__restrict__ jstar,
                                             const int32_t *__restrict__ sbest, u64 *__restrict__ win,
                                             int32_t *__restrict__ grp, uint8_t *__restrict__ merged, int h, int i,
                                             int l16) {
    // everything addressed by the token first (one round trip), then the matched slot's key row
    const size_t ti = (size_t)h * n_new + i;
    verify_core<BF16, D>(K, K_new, cp + ti * r, r, C, n_new, qscale, metric, tau2_q16, win, grp, merged, h, i, l16,
                         jstar[ti], sbest[ti]);
}

// ---- plan ----------------------------------------------------------------------------------------------
// NB + 1 workgroups of PLAN_THREADS threads per head (grid (NB + 1) x H).  The last one ranks the unmerged tokens.
// Each of the others counts the unmerged tokens and so knows e, the number of evictions needed.  When e > 0 they
// split the slots into NB contiguous ranges and find the e oldest untouched slots together:
//   threshold key T and the number of ties to take -> counts per workgroup -> ordered compaction, victims in
//   ascending slot order.
// T is normally read off the age histogram the verify launch left (no communication); otherwise: range of the keys ->
// histogram over that range (1024 bins, a second one inside the threshold bin when the range is wider).
// Between phases the workgroups of a head meet at a counter in global memory (head_barrier).  The grid is
// kept small enough (NB * H <= PLAN_MAX_GRID workgroups of 256 threads) to be resident at once, and every wait
// is bounded: a wait that runs out raises stats[7] and lets the kernel finish.
constexpr int PLAN_THREADS = 256;
constexpr int PLAN_WAVES = PLAN_THREADS / 64;
constexpr int PLAN_NB_MAX = 16;
constexpr int PLAN_MAX_GRID = 1024;
constexpr int PLAN_BINS = 1024;
constexpr int PLAN_SPIN_LIMIT = 1 << 20;
// per-head scratch in global memory (32-bit words), zeroed by the encode launch
constexpr int PS_BAR = 0;                       // 4 arrival counters
constexpr int PS_MAXK = 4, PS_MAXNK = 5;        // max key, max ~key
constexpr int PS_TOT = 6, PS_ERR = 7;           // eligible slots, bounded wait ran out
constexpr int PS_BLK = 8;                       // per workgroup, 64 bits: valid | count key > T | count key == T
constexpr int PS_FUT = 40;                      // some live slot carries a stamp above this call's frame id
constexpr int PS_HIST = 64;                     // histograms of PLAN_BINS: ages (from the verify launch), two select levels
constexpr int PS_STRIDE = PS_HIST + 3 * PLAN_BINS;
static_assert(PS_STRIDE == PLAN_SCRATCH_WORDS, "workspace layout");

__device__ __forceinline__ unsigned ld_agent(const unsigned *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// How long the plan's workgroups wait for each other, and for how many arrivals: normally PLAN_SPIN_LIMIT rounds for the
// head's own workgroups; the test hook fastar_debug_plan_wait shortens the wait and adds arrivals that never come, so
// that the exit of a wait that runs out can be exercised while every workgroup still finishes.
struct PlanWait {
    int spin_limit;
    unsigned extra_arrivals;
};
// All NB workgroups of a head arrive at counter *ctr; returns when all have (or the bounded wait ran out: bit 0 of *err).
// What the workgroups of a head tell each other inside this kernel goes through device-scope atomic operations only
// (additions / maxima on the head's scratch words before the meeting, atomic loads of them after it), which are performed
// at the memory side, past the per-XCD caches.  So no cache maintenance is needed, only order: every thread waits until
// its own memory operations have been acknowledged (vmcnt(0): on this architecture stores and atomics without a return
// value count there too), then the workgroup meets, then one thread announces the arrival; whoever sees all arrivals
// issues its loads after that.  A device-scope fence instead would write back and invalidate the XCD's L2 (dirty lines of
// the launches before included): measured 10 - 15 us per meeting here.
__device__ __forceinline__ void head_barrier(unsigned *ctr, unsigned nb, unsigned *err, PlanWait pw) {
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    __syncthreads();
    if (nb > 1 && threadIdx.x == 0) {
        atomicAdd(ctr, 1u);
        int spins = 0;
        while (ld_agent(ctr) < nb + pw.extra_arrivals) {
            if (++spins > pw.spin_limit) {
                atomicOr(err, 1u);
                break;
            }
            __builtin_amdgcn_s_sleep(4);
        }
    }
    __syncthreads();
}

// Block-wide ordered exclusive prefix over the threads, for a flag or a per-thread count.
struct BlockScan {
    unsigned *wtot;  // [PLAN_WAVES] in LDS
    __device__ __forceinline__ unsigned excl(bool flag, unsigned &total) {
        const int lane = lane_id(), wave = threadIdx.x >> 6;
        const unsigned long long m = __ballot(flag);
        __syncthreads();  // previous use of wtot finished
        if (lane == 0) wtot[wave] = __popcll(m);
        __syncthreads();
        unsigned pos = __popcll(m & ((1ull << lane) - 1ull));
        total = 0;
#pragma unroll
        for (int w = 0; w < PLAN_WAVES; ++w) {
            const unsigned c = wtot[w];
            if (w < wave) pos += c;
            total += c;
        }
        return pos;
    }
    __device__ __forceinline__ unsigned excl_sum(unsigned v, unsigned &total) {
        const int lane = lane_id(), wave = threadIdx.x >> 6;
        unsigned incl = v;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const unsigned o = __shfl_up(incl, off, WAVE);
            if (lane >= off) incl += o;
        }
        __syncthreads();
        if (lane == 63) wtot[wave] = incl;
        __syncthreads();
        unsigned pos = incl - v;
        total = 0;
#pragma unroll
        for (int w = 0; w < PLAN_WAVES; ++w) {
            const unsigned c = wtot[w];
            if (w < wave) pos += c;
            total += c;
        }
        return pos;
    }
    __device__ __forceinline__ unsigned sum(unsigned v) {
        unsigned tot;
        excl_sum(v, tot);
        return tot;
    }
};

// PLAN_TOK_MAX: tokens per thread kept in registers (8: frames up to 2048 tokens; 16: up to 4096; longer frames are
// re-read from memory in dependent loads).

// PLAN_PER_MAX: slots per thread kept in registers (longer runs are re-read from memory); 16 for caches up to
// 16 * 256 * NB slots per head, 64 beyond (a 64-frame world-model cache: 57 slots per thread).
template <int PLAN_PER_MAX, int PLAN_TOK_MAX>
__global__ __launch_bounds__(PLAN_THREADS) void tc_plan_kernel(const int32_t *__restrict__ len,
                                                               const int32_t *__restrict__ stamp, int C, int n_new,
                                                               int frame_id, const int32_t *__restrict__ jstar,
                                                               const uint8_t *__restrict__ merged,
                                                               const u64 *__restrict__ win, int32_t *__restrict__ rank,
                                                               int32_t *__restrict__ victims, int32_t *__restrict__ hs,
                                                               int32_t *__restrict__ stats, unsigned *__restrict__ ps_all,
                                                               int ws_persistent, int self_hist, PlanWait pw) {
    extern __shared__ unsigned touched[];  // bitmap over this workgroup's slot range
    __shared__ unsigned lhist[PLAN_BINS];
    __shared__ unsigned wtot[PLAN_WAVES];
    __shared__ unsigned red_a[PLAN_WAVES], red_b[PLAN_WAVES];
    __shared__ unsigned sh_bin, sh_above;
    __shared__ unsigned sh_blk[2 * PLAN_NB_MAX];
    static_assert(PLAN_THREADS * 4 == PLAN_BINS, "one thread per four bins");
    const int h = blockIdx.y, b = blockIdx.x, NB = gridDim.x - 1;  // the last workgroup of a head only ranks
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const int L = min(len[h], C);
    unsigned *ps = ps_all + (size_t)h * PS_STRIDE;
    BlockScan scan{wtot};
    const size_t tb = (size_t)h * n_new, cb = (size_t)h * C;

    // workgroup NB of every head only ranks the unmerged tokens, ascending token order
    if (b == NB) {
        unsigned done = 0;
        for (int base = 0; base < n_new; base += PLAN_THREADS) {
            const int i = base + tid;
            const bool unm = i < n_new && merged[tb + i] == 0;
            unsigned tot;
            const unsigned pos = scan.excl(unm, tot);
            if (i < n_new) rank[tb + i] = unm ? (int)(done + pos) : -1;
            done += tot;
        }
        return;
    }
    // First round of loads, all independent: the tokens' merge flags and slots (PLAN_TOK_MAX per thread in
    // registers), this thread's run of stamps, four bins of the age histogram.
    const int32_t *st = stamp + cb;
    int tj[PLAN_TOK_MAX];  // slot a token merged into, -1: not merged (or beyond n_new)
    const bool tok_cached = n_new <= PLAN_TOK_MAX * PLAN_THREADS;
    unsigned n_unm;
    {
        unsigned c = 0;
        if (tok_cached) {
            unsigned char mg[PLAN_TOK_MAX];
#pragma unroll
            for (int k = 0; k < PLAN_TOK_MAX; ++k) {
                const int i = tid + k * PLAN_THREADS;
                mg[k] = i < n_new ? merged[tb + i] : 1;
                tj[k] = i < n_new ? jstar[tb + i] : -1;
            }
#pragma unroll
            for (int k = 0; k < PLAN_TOK_MAX; ++k) {
                c += mg[k] == 0 ? 1u : 0u;
                if (!mg[k] || tid + k * PLAN_THREADS >= n_new) tj[k] = -1;
            }
        } else {
            for (int i = tid; i < n_new; i += PLAN_THREADS) c += merged[tb + i] == 0 ? 1u : 0u;
        }
        // the loads below do not depend on the count: issued before the reduction waits for the ones above
        n_unm = c;
    }
    // Long runs (PLAN_PER_MAX 64) start on multiples of four slots so that their stamps can be read 16 bytes at a time.
    // A thread's run is contiguous, so a load in which every lane reads from its own run touches 64 cache lines: the runs
    // of a wavefront (contiguous too) are instead read in four pieces of 16 runs each, consecutive lanes consecutive
    // 16 bytes, and handed to their owners through a piece of LDS that belongs to the wavefront.
    constexpr bool QUADS = PLAN_PER_MAX > 16;
    __shared__ __attribute__((aligned(16))) int stage[QUADS ? PLAN_WAVES * 16 * PLAN_PER_MAX : 4];
    const int span = QUADS ? (((L + NB - 1) / NB + 3) & ~3) : (L + NB - 1) / NB;
    const int s0 = min(b * span, L), s1 = min(s0 + span, L);
    const int per_raw = (span + PLAN_THREADS - 1) / PLAN_THREADS;
    const int per = QUADS ? ((per_raw + 3) & ~3) : per_raw;
    const int j0 = min(s0 + tid * per, s1), j1 = min(j0 + per, s1);
    const bool maybe = L + n_new > C;  // uniform: otherwise no eviction can be needed
    const bool cached = per <= PLAN_PER_MAX;
    int sreg[PLAN_PER_MAX];
    unsigned hreg[4] = {0, 0, 0, 0};
    if (maybe) {
        if (cached && QUADS && (((uintptr_t)st & 15) == 0)) {
            int *wst = stage + wave * (16 * PLAN_PER_MAX);   // this wavefront's piece: 16 runs
            const int piece = 16 * per;                       // slots of 16 runs: at most 1024, i.e. four 16-byte loads per lane
            const int wbase = s0 + wave * 64 * per;           // first slot of the wavefront's runs (may lie beyond s1)
            auto load_piece = [&](int c, i32x4 (&v)[4]) {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int q = u * 64 + lane;              // quad of the piece
                    const int slot = wbase + c * piece + 4 * q;
                    v[u] = i32x4{0, 0, 0, 0};
                    if (4 * q < piece) {
                        if (slot + 3 < s1) {
                            v[u] = *(const i32x4 *)(st + slot);
                        } else {
#pragma unroll
                            for (int e = 0; e < 4; ++e) v[u][e] = slot + e < s1 ? st[slot + e] : 0;
                        }
                    }
                }
            };
            i32x4 cur[4], nxt[4];
            load_piece(0, cur);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (c + 1 < 4) load_piece(c + 1, nxt);        // in flight while this piece is handed over
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int q = u * 64 + lane;
                    if (4 * q < piece) *(i32x4 *)(wst + 4 * q) = cur[u];
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                if ((lane >> 4) == c) {                       // the owners of this piece's runs
                    const int *mine = wst + (lane & 15) * per;
#pragma unroll
                    for (int k = 0; k < PLAN_PER_MAX; k += 4) {
                        if (k < per) {
                            const i32x4 w = *(const i32x4 *)(mine + k);
                            sreg[k] = w[0]; sreg[k + 1] = w[1]; sreg[k + 2] = w[2]; sreg[k + 3] = w[3];
                        }
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
                for (int u = 0; u < 4; ++u) cur[u] = nxt[u];
            }
        } else if (cached) {
#pragma unroll
            for (int k = 0; k < PLAN_PER_MAX; ++k) sreg[k] = j0 + k < j1 ? st[j0 + k] : 0;
        }
        if (!self_hist) {
#pragma unroll
            for (int q = 0; q < 4; ++q) hreg[q] = ps[PS_HIST + 4 * tid + q];   // written by the previous kernel
        }
    }
    n_unm = scan.sum(n_unm);
    int e = L + (int)n_unm - C;
    if (e < 0) e = 0;
    int n_victims = 0;
    if (e > 0) {  // uniform over the head's workgroups: the cache is full, evict the e oldest untouched slots
        // visit_tok(f): f(token, slot) for the merged tokens this thread looks after
        auto visit_tok = [&](auto &&f) {
            if (tok_cached) {
#pragma unroll
                for (int k = 0; k < PLAN_TOK_MAX; ++k)
                    if (tj[k] >= 0) f(tid + k * PLAN_THREADS, tj[k]);
            } else {
                for (int i = tid; i < n_new; i += PLAN_THREADS)
                    if (merged[tb + i]) f(i, jstar[tb + i]);
            }
        };
        // second round of loads: for the merged tokens, the record of their slot's group and the slot's stamp
        u64 wrec[PLAN_TOK_MAX];
        int wst[PLAN_TOK_MAX];
        if (tok_cached && !self_hist) {
#pragma unroll
            for (int k = 0; k < PLAN_TOK_MAX; ++k) {
                wrec[k] = tj[k] >= 0 ? win[cb + tj[k]] : 0ull;
                wst[k] = tj[k] >= 0 ? st[tj[k]] : 0;
            }
        }
        const int n_words = (span + 31) / 32 + 1;
        for (int w = tid; w < n_words; w += PLAN_THREADS) touched[w] = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) lhist[4 * tid + q] = hreg[q];
        __syncthreads();
        visit_tok([&](int, int j) {
            if (j >= s0 && j < s1) atomicOr(&touched[(j - s0) >> 5], 1u << ((j - s0) & 31));
        });
        __syncthreads();
        u64 elig = 0;  // bit k: slot j0 + k is live and untouched
        if (cached && j0 < j1) {   // the run's bits of the bitmap: 64 bits from bit j0 - s0 on, out of three words
            const int o = j0 - s0, w0 = o >> 5, sh = o & 31;
            u64 t = (u64)touched[w0] | ((u64)touched[w0 + 1] << 32);
            if (sh) t = (t >> sh) | ((u64)touched[w0 + 2] << (64 - sh));
            const int n = j1 - j0;
            elig = ~t & (n >= 64 ? ~0ull : ((1ull << n) - 1ull));
        }
        // visit(f): f(slot, key) for the eligible slots of this thread's run, ascending; key: larger = older
        auto visit = [&](auto &&f) {
            if (cached) {
#pragma unroll
                for (int k = 0; k < PLAN_PER_MAX; ++k)
                    if ((elig >> k) & 1ull) f(j0 + k, ~((unsigned)sreg[k] ^ 0x80000000u));
            } else {
                for (int j = j0; j < j1; ++j)
                    if (!((touched[(j - s0) >> 5] >> ((j - s0) & 31)) & 1u)) f(j, ~((unsigned)st[j] ^ 0x80000000u));
            }
        };
        // thread t owns the four bins 1023-4t .. 1020-4t of a histogram gh in global memory (descending keys):
        // finds the bin in which the want-th largest entry lies and the number of entries above that bin
        auto search = [&](const unsigned (&c4)[4], unsigned want, unsigned &total, unsigned &bin, unsigned &above) {
            const unsigned mine = c4[0] + c4[1] + c4[2] + c4[3];
            unsigned before = scan.excl_sum(mine, total);
            if (tid == 0) sh_bin = 0xFFFFFFFFu;
            __syncthreads();
            if (before < want && want <= before + mine) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    if (before < want && want <= before + c4[q]) {
                        sh_bin = PLAN_BINS - 1 - (4 * tid + q);
                        sh_above = before;
                    }
                    before += c4[q];
                }
            }
            __syncthreads();
            bin = sh_bin;
            above = sh_above;
            __syncthreads();
        };
        bool take_all = false;
        unsigned T = 0, need = (unsigned)e, cnt_el = 0;
        // Fast path: the verify launch left the histogram of all live slots' ages; subtract the slots touched in this
        // frame (each counted once, by the token that represents its group) and read the threshold off it.  Every
        // workgroup does this on the same data, so no meeting is needed.  It does not apply when a stamp lies in
        // the future or the threshold falls into the last bin (ages >= 1023 lumped together).
        // With self_hist the launch before left no histogram (a long cache: reading every stamp there as well costs more
        // than one meeting here): every workgroup counts the ages of its eligible slots from the stamps it holds, a run of
        // equal ages with one addition, the head's workgroups add their bins up in global memory and meet once.
        bool fast = self_hist ? true : ps[PS_FUT] == 0u;   // written by the previous kernel
        unsigned c4[4] = {0u, 0u, 0u, 0u};
        if (fast) {
            if (self_hist) {
                bool future = false;
                unsigned run_bin = 0u, run_n = 0u;
                visit([&](int, unsigned u) {
                    const int sv = (int)(~u ^ 0x80000000u);   // the stamp behind the key
                    future = future || sv > frame_id;
                    const unsigned bin = min((unsigned)frame_id - (unsigned)sv, (unsigned)(PLAN_BINS - 1));
                    if (bin != run_bin && run_n) {
                        atomicAdd(&lhist[run_bin], run_n);
                        run_n = 0u;
                    }
                    run_bin = bin;
                    run_n += 1u;
                });
                if (run_n) atomicAdd(&lhist[run_bin], run_n);
                __syncthreads();
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (lhist[4 * tid + q]) atomicAdd(&ps[PS_HIST + 4 * tid + q], lhist[4 * tid + q]);
                if (__any(future) && lane == 0) atomicOr(&ps[PS_FUT], 1u);
                head_barrier(&ps[PS_BAR + 3], NB, &ps[PS_ERR], pw);
#pragma unroll
                for (int q = 0; q < 4; ++q) c4[q] = ld_agent(&ps[PS_HIST + PLAN_BINS - 1 - (4 * tid + q)]);
                fast = ld_agent(&ps[PS_FUT]) == 0u;   // uniform over the head
            } else {
            if (tok_cached) {
#pragma unroll
                for (int k = 0; k < PLAN_TOK_MAX; ++k)
                    if (tj[k] >= 0 && (int)(0xFFFFFFFFu - (unsigned)wrec[k]) == tid + k * PLAN_THREADS) {
                        const unsigned age = (unsigned)frame_id - (unsigned)wst[k];
                        atomicSub(&lhist[min(age, (unsigned)(PLAN_BINS - 1))], 1u);
                    }
            } else {
                visit_tok([&](int i, int j) {
                    if ((int)(0xFFFFFFFFu - (unsigned)win[cb + j]) == i) {
                        const unsigned age = (unsigned)frame_id - (unsigned)st[j];
                        atomicSub(&lhist[min(age, (unsigned)(PLAN_BINS - 1))], 1u);
                    }
                });
            }
            __syncthreads();
#pragma unroll
            for (int q = 0; q < 4; ++q) c4[q] = lhist[PLAN_BINS - 1 - (4 * tid + q)];
            }
        }
        if (fast) {
            unsigned bin, above;
            search(c4, (unsigned)e, cnt_el, bin, above);
            take_all = cnt_el <= (unsigned)e;
            if (!take_all) {
                if (bin >= (unsigned)(PLAN_BINS - 1)) {
                    fast = false;
                } else {
                    T = ~((unsigned)(frame_id - (int)bin) ^ 0x80000000u);  // key of the stamp frame_id - bin
                    need = (unsigned)e - above;
                }
            }
        }
        if (!fast) {
            // General path: range of the keys and number of eligible slots over the whole head, then a histogram
            // select on that range (a second histogram inside the threshold bin when the range is wider than the
            // bins), the workgroups of the head meeting between the steps.
            {
                unsigned kmin = 0xFFFFFFFFu, kmax = 0u, c = 0u;
                visit([&](int, unsigned u) {
                    kmin = min(kmin, u);
                    kmax = max(kmax, u);
                    c += 1;
                });
#pragma unroll
                for (int off = 32; off >= 1; off >>= 1) {
                    kmin = min(kmin, shfl_xor(kmin, off));
                    kmax = max(kmax, shfl_xor(kmax, off));
                }
                if (lane == 0) {
                    red_a[wave] = kmin;
                    red_b[wave] = kmax;
                }
                c = scan.sum(c);  // its barriers also publish red_a / red_b
                if (tid == 0 && c > 0) {
                    kmin = 0xFFFFFFFFu;
                    kmax = 0u;
                    for (int w = 0; w < PLAN_WAVES; ++w) {
                        kmin = min(kmin, red_a[w]);
                        kmax = max(kmax, red_b[w]);
                    }
                    atomicMax(&ps[PS_MAXK], kmax);
                    atomicMax(&ps[PS_MAXNK], ~kmin);
                    atomicAdd(&ps[PS_TOT], c);
                }
            }
            head_barrier(&ps[PS_BAR + 0], NB, &ps[PS_ERR], pw);
            const unsigned umax = ld_agent(&ps[PS_MAXK]), umin = ~ld_agent(&ps[PS_MAXNK]);
            cnt_el = ld_agent(&ps[PS_TOT]);
            take_all = cnt_el <= (unsigned)e;  // fewer eligible slots than evictions needed: take them all
            T = umax;
            need = (unsigned)e;
            if (!take_all) {
                // Among the keys in [lo, lo + width), with `want` of them to take from the top: histogram over the
                // head (bin = (key - lo) >> sh), then the bin in which the want-th largest key lies.
                auto level = [&](unsigned lo, unsigned width, int sh, unsigned want, int which, unsigned &bin, unsigned &above) {
                    for (int k = tid; k < PLAN_BINS; k += PLAN_THREADS) lhist[k] = 0;
                    __syncthreads();
                    visit([&](int, unsigned u) {
                        const unsigned rel = u - lo;
                        if (u >= lo && rel < width && (rel >> sh) < (unsigned)PLAN_BINS) atomicAdd(&lhist[rel >> sh], 1u);
                    });
                    __syncthreads();
                    unsigned *gh = ps + PS_HIST + (1 + which) * PLAN_BINS;
                    for (int k = tid; k < PLAN_BINS; k += PLAN_THREADS)
                        if (lhist[k]) atomicAdd(&gh[k], lhist[k]);
                    head_barrier(&ps[PS_BAR + 1 + which], NB, &ps[PS_ERR], pw);
                    unsigned c4[4], total;
#pragma unroll
                    for (int q = 0; q < 4; ++q) c4[q] = ld_agent(&gh[PLAN_BINS - 1 - (4 * tid + q)]);
                    search(c4, want, total, bin, above);
                };
                const unsigned range = umax - umin;
                int sh = 0;
                while ((range >> sh) >= (unsigned)PLAN_BINS) ++sh;
                unsigned bin, above;
                level(umin, 0xFFFFFFFFu, sh, (unsigned)e, 0, bin, above);
                if (sh == 0) {
                    T = umin + bin;
                    need = (unsigned)e - above;
                } else {  // resolve inside the coarse bin (ranges up to 2^20 frames; wider ones are not resolved exactly)
                    const unsigned lo2 = umin + (bin << sh);
                    const int sh2 = sh > 10 ? sh - 10 : 0;
                    if (sh2 > 0 && tid == 0) atomicOr(&ps[PS_ERR], 2u);
                    unsigned bin2, above2;
                    level(lo2, 1u << sh, sh2, (unsigned)e - above, 1, bin2, above2);
                    T = lo2 + (bin2 << sh2);
                    need = (unsigned)e - above - above2;
                }
            }
        }
        n_victims = take_all ? (int)cnt_el : e;
        // counts per workgroup, the workgroups meet, then ordered compaction: victims in ascending slot order
        unsigned c_gt = 0, c_eq = 0;
        visit([&](int, unsigned u) {
            c_gt += (take_all || u > T) ? 1u : 0u;
            c_eq += (!take_all && u == T) ? 1u : 0u;
        });
        unsigned blk_gt, blk_eq;
        scan.excl_sum(c_gt, blk_gt);
        const unsigned eq_base_thr = scan.excl_sum(c_eq, blk_eq);
        // Publish this workgroup's counts as one 64-bit word with a valid bit, then wait (bounded) for the words of
        // the workgroups below: only those are needed for the positions, and the wait doubles as the read.
        u64 *blk = (u64 *)(ps + PS_BLK);
        if (tid == 0)
            __hip_atomic_store(&blk[b], (1ull << 63) | ((u64)blk_gt << 32) | (u64)blk_eq, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        if (tid < b) {
            u64 v = 0;
            int spins = 0;
            while (!((v = __hip_atomic_load(&blk[tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) >> 63)) {
                if (++spins > pw.spin_limit) {
                    atomicOr(&ps[PS_ERR], 1u);
                    break;
                }
                __builtin_amdgcn_s_sleep(2);
            }
            sh_blk[2 * tid] = (unsigned)(v >> 32) & 0x7FFFFFFFu;
            sh_blk[2 * tid + 1] = (unsigned)v;
        }
        __syncthreads();
        unsigned pos_base = 0, eq_before = 0;
        for (int bb = 0; bb < b; ++bb) {
            const unsigned g = sh_blk[2 * bb], q = sh_blk[2 * bb + 1];
            const unsigned tk = eq_before >= need ? 0u : min(q, need - eq_before);
            pos_base += g + tk;
            eq_before += q;
        }
        const unsigned eq_blk_take = eq_before >= need ? 0u : min(blk_eq, need - eq_before);  // ties this workgroup takes
        const unsigned eq_take = eq_base_thr >= eq_blk_take ? 0u : min(c_eq, eq_blk_take - eq_base_thr);
        unsigned tot;
        unsigned pos = pos_base + scan.excl_sum(c_gt + eq_take, tot);
        unsigned eq_seen = 0;
        visit([&](int j, unsigned u) {
            bool take = take_all || u > T;
            if (!take_all && u == T) {
                take = eq_seen < eq_take;
                eq_seen += 1;
            }
            if (take) {
                if (pos < (unsigned)n_new) victims[tb + pos] = j;
                pos += 1;
            }
        });
    }
    if (b == 0 && tid == 0) {
        const int n_dropped = e - n_victims;
        const int n_app = (int)n_unm - n_dropped;
        const int newL = L + n_app - n_victims;
        int32_t *o = hs + (size_t)h * HS_STRIDE;
        const int mark = o[7];
        o[0] = L; o[1] = (int)n_unm; o[2] = e; o[3] = n_victims; o[4] = n_dropped; o[5] = newL;
        int32_t *s = stats + (size_t)h * 8;
        s[0] = newL; s[1] = n_new - (int)n_unm; s[2] = n_app; s[3] = n_victims; s[4] = n_dropped;
        // bit 0 of the error word (a wait ran out) may still be raised by a workgroup that finishes later: the apply
        // launch looks again and, if it is set, leaves the head's cache as it was
        const unsigned err = e > 0 ? ld_agent(&ps[PS_ERR]) : 0u;
        int status = (err & 1u) ? 1 : (err & 2u) ? 2 : 0;
        // a workspace declared persistent must be a zero-filled one or one a finished call left behind
        if (ws_persistent && mark != 0 && mark != WS_CLEAN) status = 3;
        o[6] = status == 3 ? 3 : 0;   // for the apply launch: records and scratch of this workspace mean nothing
        s[5] = 0; s[6] = 0; s[7] = status;
    }
}

// workgroups per head of tc_plan_kernel and its dynamic LDS (the touched bitmap of one workgroup's slot range).
// The workgroups of a head wait for each other, so the whole grid has to be resident at once.  What a compute unit
// holds of the kernel's instantiations without dynamic LDS (registers, wavefront slots) and the number of compute units
// are asked of the runtime once per device; with LDS (bitmap + about 5 KB of static arrays) fewer may fit its 160 KB.
// The grid (nb + 1) * H stays within that (and within PLAN_MAX_GRID).
struct PlanResidency {
    int per_cu, n_cu;
};
static int plan_residency(PlanResidency *out) {
    static DeviceOnce once;
    static PlanResidency table[DeviceOnce::MAX_DEVICES];
    const int rc = once.run([](int dev) {
        int least = INT_MAX, n_cu = 0;
        const void *kernels[4] = {(const void *)tc_plan_kernel<64, 16>, (const void *)tc_plan_kernel<64, 8>,
                                  (const void *)tc_plan_kernel<16, 16>, (const void *)tc_plan_kernel<16, 8>};
        for (const void *k : kernels) {
            int n = 0;
            if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, k, PLAN_THREADS, 0) != hipSuccess) return FASTAR_ERR_HIP;
            least = std::min(least, n);
        }
        if (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return FASTAR_ERR_HIP;
        if (least < 1 || n_cu < 1) return FASTAR_ERR_HIP;
        table[dev] = {least, n_cu};
        return FASTAR_OK;
    });
    if (rc != FASTAR_OK) return rc;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return FASTAR_ERR_HIP;
    *out = table[dev];
    return FASTAR_OK;
}
static int plan_residency_setup() {
    PlanResidency pr;
    return plan_residency(&pr);
}
static size_t plan_lds_bytes(int C, int nb) { return ((size_t)((C + nb - 1) / nb + 3 + 31) / 32 + 2) * 4; }
static int plan_nb(int H, int C, PlanResidency pr) {
    int nb = (C + 2047) / 2048;
    if (nb > PLAN_NB_MAX) nb = PLAN_NB_MAX;
    if (nb < 1) nb = 1;
    for (; nb > 1; --nb) {
        // static arrays: about 5 KB, and 16 KB more in the instantiation for long runs (the hand-over area of the stamps)
        const bool long_runs = ((C + nb - 1) / nb + PLAN_THREADS - 1) / PLAN_THREADS > 16;
        const size_t lds = plan_lds_bytes(C, nb) + (long_runs ? 21 : 5) * 1024;
        size_t per_cu = (size_t)160 * 1024 / lds;
        if (per_cu > (size_t)pr.per_cu) per_cu = (size_t)pr.per_cu;
        size_t resident = per_cu * (size_t)pr.n_cu;
        if (resident > (size_t)PLAN_MAX_GRID) resident = PLAN_MAX_GRID;
        if ((size_t)(nb + 1) * (size_t)H <= resident) break;
    }
    return nb;
}

// ---- apply ---------------------------------------------------------------------------------------------
template <bool BF16, int D>
__global__ __launch_bounds__(256) void tc_apply_kernel(void *__restrict__ K, void *__restrict__ V, int8_t *__restrict__ code,
                                                       int32_t *__restrict__ cnt, int32_t *__restrict__ stamp, int C,
                                                       int r, const void *__restrict__ K_new,
                                                       const void *__restrict__ V_new, const int8_t *__restrict__ ck,
                                                       int n_new, int frame_id, const int32_t *__restrict__ jstar,
                                                       const uint8_t *__restrict__ merged, u64 *win, int32_t *grp,
                                                       const int32_t *__restrict__ rank,
                                                       const int32_t *__restrict__ victims, int32_t *hs,
                                                       int32_t *__restrict__ merge_map, int32_t *__restrict__ len,
                                                       int rep_mode, unsigned *__restrict__ ps_all, int ps_words,
                                                       int32_t *__restrict__ stats) {
    typedef RowPiece<BF16, D> RP;
    const int h = blockIdx.y;
    // A wait of the plan ran out for this head (bit 0 of its error word; every workgroup of this launch sees it, because
    // none clears the scratch words then): the victims are not to be trusted, so nothing of the head is applied.  Its
    // cache stays as it was before the call, every token counts as dropped, and the workspace is marked as not clean.
    // The same when the workspace was declared persistent but is neither zero-filled nor left by a finished call
    // (status 3, word 6 of the head's scalars): its records mean nothing.
    const bool ws_dirty = hs[(size_t)h * HS_STRIDE + 6] == 3;
    if (ws_dirty || (ps_all[(size_t)h * ps_words + PS_ERR] & 1u)) {
        if (blockIdx.x == 0 && threadIdx.x == 0) {
            int32_t *s = stats + (size_t)h * 8;
            s[0] = hs[(size_t)h * HS_STRIDE + 0]; s[1] = 0; s[2] = 0; s[3] = 0; s[4] = n_new; s[5] = 0; s[6] = 0;
            s[7] = ws_dirty ? 3 : 1;
            if (!ws_dirty) hs[(size_t)h * HS_STRIDE + 7] = WS_FAILED;
        }
        const int i = blockIdx.x * (blockDim.x / 16) + (threadIdx.x >> 4);
        if (i < n_new && (threadIdx.x & 15) == 0) {
            merge_map[(size_t)h * n_new + i] = -1;
            const_cast<uint8_t *>(merged)[(size_t)h * n_new + i] = 0;
        }
        return;
    }
    // the new length is published here and not by the plan: its workgroups read len[h] at different times
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        len[h] = hs[(size_t)h * HS_STRIDE + 5];
        hs[(size_t)h * HS_STRIDE + 7] = WS_CLEAN;   // with the two clean-ups below: the workspace is left as a zero-filled one
    }
    // the plan is done with its scratch words: cleared for the next call that shares this workspace
    for (int k = blockIdx.x * blockDim.x + threadIdx.x; k < ps_words; k += gridDim.x * blockDim.x)
        ps_all[(size_t)h * ps_words + k] = 0u;
    const int l16 = threadIdx.x & 15;
    const int sub = (threadIdx.x & 63) >> 4;  // which 16-lane group of the wavefront
    const int i = blockIdx.x * (blockDim.x / 16) + (threadIdx.x >> 4);
    if (i >= n_new) return;
    const size_t tb = (size_t)h * n_new, ti = tb + i, cb = (size_t)h * C;
    const int32_t *o = hs + (size_t)h * HS_STRIDE;
    const int L = o[0], n_unm = o[1], n_victims = o[3], n_dropped = o[4];
    // First round of loads, all addressed by the token: flags, destination data, and the token's own rows (bit
    // copies).  The second round (records and value row of the slot, or the victim slot) depends on them.
    const bool mg = merged[ti] != 0;
    const int j = jstar[ti];
    const int a = rank[ti];
    typename RP::Raw kraw = RP::load_raw(K_new, ti, l16), vraw = RP::load_raw(V_new, ti, l16);
    unsigned cw = 0;
    if (l16 < r / 4) cw = ((const unsigned *)(ck + ti * r))[l16];
    int dst = -1;
    if (mg) {
        dst = j;
        // second round of loads, everything addressed by the slot at once: its records and multiplicity, and already
        // its value row (and key row for the mean key), which only the group's representative goes on to use
        const bool mean_key = rep_mode == 1;
        float acc[RP::EPL], vn[RP::EPL], kacc[RP::EPL], kn[RP::EPL];
        const u64 wkey = win[cb + j];
        const int gc = grp[cb + j];
        const int m0 = cnt[cb + j];
        RP::load(V, cb + j, l16, acc);
        if (mean_key) RP::load(K, cb + j, l16, kacc);
        const int widx = (int)(0xFFFFFFFFu - (unsigned)wkey);
        if (widx == i) {  // this token represents the group: it refreshes the slot
            // ... and clears the group's records behind it: the other joiners only look for their own index in the
            // record, which neither the old nor the cleared value shows them
            if (l16 == 0) {
                win[cb + j] = 0;
                grp[cb + j] = 0;
            }
            // mean value; with rep_mode 1 also the mean key, whose stored bits feed later integer decisions: single
            // float32 operations in a fixed order (multiplicity * old row, members in ascending token order, one division)
#pragma unroll
            for (int e = 0; e < RP::EPL; ++e) acc[e] *= (float)m0;
            if (mean_key) {
#pragma unroll
                for (int e = 0; e < RP::EPL; ++e) kacc[e] = __fmul_rn((float)m0, kacc[e]);
            }
            if (gc == 1) {
                RP::unpack(vraw, vn);
#pragma unroll
                for (int e = 0; e < RP::EPL; ++e) acc[e] += vn[e];
                if (mean_key) {
                    RP::unpack(kraw, kn);
#pragma unroll
                    for (int e = 0; e < RP::EPL; ++e) kacc[e] = __fadd_rn(kacc[e], kn[e]);
                }
            } else {  // several joiners: add their rows in ascending token order
                for (int base = 0; base < n_new; base += 16) {
                    const int t = base + l16;
                    const bool member = t < n_new && merged[tb + t] && jstar[tb + t] == j;
                    unsigned mm = (unsigned)((__ballot(member) >> (16 * sub)) & 0xFFFFull);
                    while (mm) {
                        const int bit = __ffs(mm) - 1;
                        mm &= mm - 1;
                        RP::load(V_new, tb + base + bit, l16, vn);
#pragma unroll
                        for (int e = 0; e < RP::EPL; ++e) acc[e] += vn[e];
                        if (mean_key) {
                            RP::load(K_new, tb + base + bit, l16, kn);
#pragma unroll
                            for (int e = 0; e < RP::EPL; ++e) kacc[e] = __fadd_rn(kacc[e], kn[e]);
                        }
                    }
                }
            }
#pragma unroll
            for (int e = 0; e < RP::EPL; ++e) acc[e] = __fdiv_rn(acc[e], (float)(m0 + gc));
            RP::store(V, cb + j, l16, acc);
            if (mean_key) {   // the slot's code follows in tc_recode_kernel, from the stored row
#pragma unroll
                for (int e = 0; e < RP::EPL; ++e) kacc[e] = __fdiv_rn(kacc[e], (float)(m0 + gc));
                RP::store(K, cb + j, l16, kacc);
            } else if (rep_mode == 2) {
                // Medoid key: of {stored key (weight m0), joiners (weight 1)} the member x with the smallest
                // cost(x) = sum_y w_y |x - y|^2 in code space = W |x|^2 + S2 - 2 x . S1 (W = sum of the weights,
                // S1 = weighted sum of the codes, S2 = weighted sum of their squared norms): exact integers, one pass to
                // build the sums and one to evaluate the candidates (stored key first, then tokens ascending; a later
                // candidate wins only on a strictly smaller cost).  Lane l16 owns code word l16 (r <= 64: 16 words).
                // A single joiner never wins: cost(stored) = |d|^2 <= m0 |d|^2 = cost(joiner).
                if (gc > 1) {
                    const bool has_w = l16 < r / 4;
                    const unsigned ow = has_w ? ((const unsigned *)(code + (cb + j) * r))[l16] : 0u;
                    long long S1[4], S2 = (long long)m0 * dot4_i8(ow, ow, 0);
#pragma unroll
                    for (int k = 0; k < 4; ++k) S1[k] = (long long)m0 * (int)(signed char)(ow >> (8 * k));
                    for (int base = 0; base < n_new; base += 16) {
                        const int t = base + l16;
                        const bool member = t < n_new && merged[tb + t] && jstar[tb + t] == j;
                        unsigned mm = (unsigned)((__ballot(member) >> (16 * sub)) & 0xFFFFull);
                        while (mm) {
                            const int bit = __ffs(mm) - 1;
                            mm &= mm - 1;
                            const unsigned w = has_w ? ((const unsigned *)(ck + (tb + base + bit) * r))[l16] : 0u;
                            S2 += dot4_i8(w, w, 0);
#pragma unroll
                            for (int k = 0; k < 4; ++k) S1[k] += (int)(signed char)(w >> (8 * k));
                        }
                    }
                    const long long W = (long long)m0 + gc;
                    auto group16_sum64 = [](long long v) -> long long {
#pragma unroll
                        for (int off = 1; off < 16; off <<= 1) {
                            const unsigned lo = shfl_xor((unsigned)v, off), hi = shfl_xor((unsigned)((unsigned long long)v >> 32), off);
                            v += (long long)(((unsigned long long)hi << 32) | lo);
                        }
                        return v;
                    };
                    auto cost_of = [&](unsigned w) -> long long {   // this lane's share of W |x|^2 + S2 - 2 x . S1
                        long long c = W * dot4_i8(w, w, 0) + S2;
#pragma unroll
                        for (int k = 0; k < 4; ++k) c -= 2 * S1[k] * (int)(signed char)(w >> (8 * k));
                        return c;
                    };
                    long long best_cost = group16_sum64(cost_of(ow));
                    int best = -1;   // the stored key
                    for (int base = 0; base < n_new; base += 16) {
                        const int t = base + l16;
                        const bool member = t < n_new && merged[tb + t] && jstar[tb + t] == j;
                        unsigned mm = (unsigned)((__ballot(member) >> (16 * sub)) & 0xFFFFull);
                        while (mm) {
                            const int bit = __ffs(mm) - 1;
                            mm &= mm - 1;
                            const unsigned w = has_w ? ((const unsigned *)(ck + (tb + base + bit) * r))[l16] : 0u;
                            const long long c = group16_sum64(cost_of(w));
                            if (c < best_cost) {
                                best_cost = c;
                                best = base + bit;
                            }
                        }
                    }
                    if (best >= 0) {
                        RP::copy(K, cb + j, K_new, tb + best, l16);
                        if (has_w) ((unsigned *)(code + (cb + j) * r))[l16] = ((const unsigned *)(ck + (tb + best) * r))[l16];
                    }
                }
            } else {
                RP::store_raw(K, cb + j, l16, kraw);
                if (l16 < r / 4) ((unsigned *)(code + (cb + j) * r))[l16] = cw;
            }
            if (l16 == 0) {
                cnt[cb + j] = m0 + gc;
                stamp[cb + j] = frame_id;
            }
        }
    } else if (a < n_unm - n_dropped) {
        dst = a < n_victims ? victims[tb + a] : L + (a - n_victims);
        // A plan whose bounded wait ran out (stats[7] = 1) may have left victim positions unwritten: whatever they
        // hold, nothing is stored outside the cache; such a token counts as not placed.
        if ((unsigned)dst >= (unsigned)C) dst = -1;
    }
    if (!mg && dst >= 0) {
        RP::store_raw(K, cb + dst, l16, kraw);
        RP::store_raw(V, cb + dst, l16, vraw);
        if (l16 < r / 4) ((unsigned *)(code + (cb + dst) * r))[l16] = cw;
        if (l16 == 0) {
            cnt[cb + dst] = 1;
            stamp[cb + dst] = frame_id;
        }
    }
    if (l16 == 0) merge_map[ti] = dst;
}

// ---- codes of the slots whose key was replaced by a mean (rep_mode 1), from the rows tc_apply_kernel stored -----
// One wavefront per 16 tokens, as in encode_kernel; every merged token encodes its slot (the joiners of one slot
// write the same bytes).
template <bool BF16, int D, int R>
__global__ __launch_bounds__(256) void tc_recode_kernel(const void *__restrict__ K, int8_t *__restrict__ code, int C,
                                                        int n_new, const int32_t *__restrict__ jstar,
                                                        const uint8_t *__restrict__ merged,
                                                        const int8_t *__restrict__ Rm, float qscale, int shift) {
    const int h = blockIdx.y;
    const int lane = lane_id();
    const int col = lane & 15, g = lane >> 4;
    const int i = blockIdx.x * 64 + (threadIdx.x >> 6) * 16 + col;
    const bool act = i < n_new && merged[(size_t)h * n_new + i] != 0;
    const int j = act ? jstar[(size_t)h * n_new + i] : 0;
    CodeMatrix<BF16, D, R> cm;
    cm.load(Rm, lane);
    const char *row = (const char *)K + ((size_t)h * C + j) * (size_t)D * (BF16 ? 2 : 4);
    i32x4 xq[D / 64];
#pragma unroll
    for (int ks = 0; ks < D / 64; ++ks) xq[ks] = load_quantised<BF16>(row, ks, g, qscale);
#pragma unroll
    for (int cb = 0; cb < R / 16; ++cb) {
        const unsigned w = cm.code_word(xq, cb, shift);
        if (act) *(unsigned *)(code + ((size_t)h * C + j) * R + cb * 16 + 4 * g) = w;
    }
}

}  // namespace fastar

using namespace fastar;

// what tc_plan_kernel's waits are bounded by (test hook below; the default is what every caller gets)
static PlanWait g_plan_wait = {PLAN_SPIN_LIMIT, 0u};

extern "C" int fastar_debug_plan_wait(int spin_limit, int extra_arrivals) {
    if (extra_arrivals < 0) return FASTAR_ERR_INVALID_ARG;
    g_plan_wait.spin_limit = spin_limit < 0 ? PLAN_SPIN_LIMIT : spin_limit;
    g_plan_wait.extra_arrivals = (unsigned)extra_arrivals;
    return FASTAR_OK;
}

extern "C" int tempcache_compress(const fastar_cache *cache, const fastar_codec *codec, const void *K_new,
                                  const void *V_new, const void *P_new, int n_new, const int32_t *cand, int n_cand,
                                  int metric, int32_t tau2_q16, int32_t frame_id, int rep_mode, int32_t *merge_map,
                                  uint8_t *merged, int32_t *stats, void *ws, size_t ws_bytes, int ws_persistent,
                                  void *stream) {
    if (!cache || !codec || !codec->R || !K_new || !V_new || !merge_map || !merged || !stats || !ws)
        return FASTAR_ERR_INVALID_ARG;
    if (!cache->K || !cache->V || !cache->code || !cache->cnt || !cache->stamp || !cache->len)
        return FASTAR_ERR_INVALID_ARG;
    const int H = cache->H, C = cache->C, d = cache->d, r = cache->r, dtype = cache->dtype;
    if (H <= 0 || C <= 0 || n_new <= 0 || (metric != 0 && metric != 1)) return FASTAR_ERR_INVALID_ARG;
    if (rep_mode != FASTAR_REP_LAST && rep_mode != FASTAR_REP_MEAN && rep_mode != FASTAR_REP_MEDOID) return FASTAR_ERR_INVALID_ARG;
    if (ws_persistent != 0 && ws_persistent != 1) return FASTAR_ERR_INVALID_ARG;
    if (tau2_q16 < 0 || tau2_q16 > 131072) return FASTAR_ERR_INVALID_ARG;
    if (cand && n_cand <= 0) return FASTAR_ERR_INVALID_ARG;
    if (codec->shift < 1 || codec->shift > 16) return FASTAR_ERR_INVALID_ARG;
    if (dtype != FASTAR_F32 && dtype != FASTAR_BF16) return FASTAR_ERR_INVALID_ARG;
    if ((d != 64 && d != 128) || (r != 32 && r != 64)) return FASTAR_ERR_UNSUPPORTED;
    PlanResidency pr;
    if (const int rc0 = plan_residency(&pr); rc0 != FASTAR_OK) return rc0;
    const int nb = plan_nb(H, C, pr);
    if (plan_lds_bytes(C, nb) > 48 * 1024) return FASTAR_ERR_UNSUPPORTED;  // eviction bitmap of a slot range lives in LDS
    // Who counts the live slots' ages for the eviction threshold.  Short caches: the verify step, whose whole grid reads
    // the stamps while the plan's few workgroups would meet for it.  Long caches (a plan thread holds more than 16 stamps,
    // and all of its run, in registers): the plan itself, from the stamps it reads anyway: a second sweep over every
    // stamp costs more than one meeting of the head's workgroups.
    const int plan_span = (((C + nb - 1) / nb) + 3) & ~3;
    const int plan_per = (((plan_span + PLAN_THREADS - 1) / PLAN_THREADS) + 3) & ~3;
    const bool long_runs = ((C + nb - 1) / nb + PLAN_THREADS - 1) / PLAN_THREADS > 16;   // the plan's instantiation with 64 stamps per thread
    const bool self_hist = long_runs && plan_per <= 64;
    if (((uintptr_t)cache->K & 15) || ((uintptr_t)cache->V & 15) || ((uintptr_t)cache->code & 15) ||
        ((uintptr_t)K_new & 15) || ((uintptr_t)V_new & 15) || ((uintptr_t)P_new & 15) || ((uintptr_t)ws & 255))
        return FASTAR_ERR_INVALID_ARG;
    const CompressWs w = compress_ws(H, C, n_new, r);
    if (ws_bytes < w.total) return FASTAR_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    char *base = (char *)ws;
    int8_t *ck = (int8_t *)(base + w.ck);
    int8_t *cp = P_new ? (int8_t *)(base + w.cp) : ck;
    u64 *best = (u64 *)(base + w.best);
    int32_t *jstar = (int32_t *)(base + w.jstar), *sbest = (int32_t *)(base + w.sbest);
    int32_t *rank = (int32_t *)(base + w.rank), *victims = (int32_t *)(base + w.victims);
    int32_t *hs = (int32_t *)(base + w.hs);
    unsigned *plan_scratch = (unsigned *)(base + w.ps);
    u64 *win = (u64 *)(base + w.win);
    int32_t *grp = (int32_t *)(base + w.grp);
    const int64_t T = (int64_t)H * n_new;

    const size_t win_lds = cand ? match_window_lds(n_cand, r) : 0;
    const bool window = cand && win_lds <= WINDOW_LDS_MAX;
    const bool fused_encode = window && !P_new;  // the match kernel encodes its own probes
    const bool fused_verify = fused_encode && ws_persistent;   // ... and verifies its matches: nothing to clear first
    if (!fused_encode) {
        const int64_t zero_words = (int64_t)((w.ps - w.best) / 8) + (int64_t)H * PLAN_SCRATCH_WORDS / 2;  // best .. end of ps
        int rc = encode_launch(K_new, dtype, T, d, codec, r, ck, best, zero_words, s);
        if (rc != FASTAR_OK) return rc;
        if (P_new) {
            rc = encode_launch(P_new, dtype, T, d, codec, r, cp, nullptr, 0, s);
            if (rc != FASTAR_OK) return rc;
        }
    }
    if (window) {
        // the whole candidate window fits one workgroup's LDS: final arg-max per token in one launch
        if (const int rc0 = tempcache_setup(); rc0 != FASTAR_OK) return rc0;
        // 256 tokens per workgroup when 64 would give more than two rounds of workgroups over the chip (the window is
        // staged once per workgroup) and the window leaves room for the wider static arrays
        const size_t per_cu = (size_t)160 * 1024 / (win_lds + 9 * 1024);
        const bool wide = fused_encode && win_lds <= wide_window_lds_max(r) &&
                          (size_t)((n_new + 63) / 64) * (size_t)H > 2 * 256 * (per_cu > 0 ? per_cu : 1);
        // With 256 tokens per workgroup a workgroup takes several blocks of tokens, one after the other, once it has
        // staged the window: as many workgroups as the chip holds at once (the staging is then paid once per resident
        // workgroup, and no round of workgroups waits for the one before it).
        int gx = wide ? (n_new + 255) / 256 : (n_new + 63) / 64;
        if (wide) {   // equal shares of whole groups of 32 tokens, none of them empty
            gx = std::min(gx, std::max(1, (int)(256 * (per_cu > 0 ? per_cu : 1)) / H));
            const int per = (((n_new + gx - 1) / gx) + 31) & ~31;
            gx = (n_new + per - 1) / per;
        }
        const dim3 grid(gx, H);
        const bool bf = dtype == FASTAR_BF16;
        const VerifyArgs va = {cache->K, tau2_q16, merged, cache->stamp, frame_id, self_hist ? -1 : PS_HIST, PS_FUT};
        int rc = FASTAR_OK;
#define FASTAR_WIN(RR, ENC, BF, DD, VER, TT)                                                                              \
    rc = launch_match_window<RR, ENC, BF, DD, VER, TT>(grid, win_lds, s, cache->code, cache->len, C, cp, n_new, cand,      \
                                                       n_cand, metric, jstar, sbest, win, grp, K_new, codec->R,            \
                                                       codec->qscale, codec->shift, ck, plan_scratch, (int)PS_STRIDE, va)
#define FASTAR_WIN_ENC(RR, BF, DD)                                                      \
    do {                                                                                \
        if (fused_verify && wide) FASTAR_WIN(RR, true, BF, DD, true, 256);              \
        else if (fused_verify) FASTAR_WIN(RR, true, BF, DD, true, 64);                  \
        else if (wide) FASTAR_WIN(RR, true, BF, DD, false, 256);                        \
        else FASTAR_WIN(RR, true, BF, DD, false, 64);                                   \
    } while (0)
        if (!fused_encode) { if (r == 32) FASTAR_WIN(32, false, true, 128, false, 64); else FASTAR_WIN(64, false, true, 128, false, 64); }
        else if (r == 32 && d == 128) { if (bf) FASTAR_WIN_ENC(32, true, 128); else FASTAR_WIN_ENC(32, false, 128); }
        else if (r == 32) { if (bf) FASTAR_WIN_ENC(32, true, 64); else FASTAR_WIN_ENC(32, false, 64); }
        else if (d == 128) { if (bf) FASTAR_WIN_ENC(64, true, 128); else FASTAR_WIN_ENC(64, false, 128); }
        else { if (bf) FASTAR_WIN_ENC(64, true, 64); else FASTAR_WIN_ENC(64, false, 64); }
#undef FASTAR_WIN_ENC
#undef FASTAR_WIN
        if (rc != FASTAR_OK) return rc;
    } else {
        const int n_pos_cap = cand ? n_cand : C;
        const int chunk = n_pos_cap <= 4096 ? 64 : 256;
        dim3 grid((n_new + 127) / 128, (n_pos_cap + chunk - 1) / chunk, H);
#define FASTAR_MATCH(RR, CH)                                                                                         \
    do {                                                                                                             \
        if (cand)                                                                                                    \
            hipLaunchKernelGGL((tc_match_kernel<RR, CH, true>), grid, dim3(256), 0, s, cache->code, cache->len, C, cp, \
                               n_new, cand, n_cand, metric, best);                                                   \
        else                                                                                                         \
            hipLaunchKernelGGL((tc_match_kernel<RR, CH, false>), grid, dim3(256), 0, s, cache->code, cache->len, C, cp, \
                               n_new, cand, n_cand, metric, best);                                                   \
    } while (0)
        if (r == 32 && chunk == 64) FASTAR_MATCH(32, 64);
        else if (r == 32) FASTAR_MATCH(32, 256);
        else if (chunk == 64) FASTAR_MATCH(64, 64);
        else FASTAR_MATCH(64, 256);
#undef FASTAR_MATCH
        FASTAR_LAUNCH_CHECK();
        hipLaunchKernelGGL(tc_prep_kernel, dim3((n_new + 255) / 256, H), dim3(256), 0, s, best, n_new, C, cand, n_cand,
                           jstar, sbest, win, grp);
        FASTAR_LAUNCH_CHECK();
    }
    const dim3 tgrid((n_new + 15) / 16, H);
    const bool bf = dtype == FASTAR_BF16;
#define FASTAR_TC(KERNEL, ...)                                                                          \
    do {                                                                                                \
        if (bf && d == 128) hipLaunchKernelGGL((KERNEL<true, 128>), tgrid, dim3(256), 0, s, __VA_ARGS__);      \
        else if (bf) hipLaunchKernelGGL((KERNEL<true, 64>), tgrid, dim3(256), 0, s, __VA_ARGS__);               \
        else if (d == 128) hipLaunchKernelGGL((KERNEL<false, 128>), tgrid, dim3(256), 0, s, __VA_ARGS__);       \
        else hipLaunchKernelGGL((KERNEL<false, 64>), tgrid, dim3(256), 0, s, __VA_ARGS__);                       \
    } while (0)
    if (!fused_verify) {
        FASTAR_TC(tc_verify_kernel, cache->K, K_new, cp, r, C, n_new, codec->qscale, metric, tau2_q16, jstar, sbest, win,
                  grp, merged, cache->len, cache->stamp, frame_id, plan_scratch, self_hist ? -1 : PS_HIST, PS_FUT, PS_STRIDE);
        FASTAR_LAUNCH_CHECK();
    }
    {
        const bool long_frame = n_new > 8 * PLAN_THREADS;
#define FASTAR_PLAN(PM, TM)                                                                                            \
    hipLaunchKernelGGL((tc_plan_kernel<PM, TM>), dim3(nb + 1, H), dim3(PLAN_THREADS), plan_lds_bytes(C, nb), s, cache->len, \
                       cache->stamp, C, n_new, frame_id, jstar, merged, win, rank, victims, hs, stats, plan_scratch,   \
                       ws_persistent, self_hist ? 1 : 0, g_plan_wait)
        if (long_runs && long_frame) FASTAR_PLAN(64, 16);
        else if (long_runs) FASTAR_PLAN(64, 8);
        else if (long_frame) FASTAR_PLAN(16, 16);
        else FASTAR_PLAN(16, 8);
#undef FASTAR_PLAN
    }
    FASTAR_LAUNCH_CHECK();
    FASTAR_TC(tc_apply_kernel, cache->K, cache->V, cache->code, cache->cnt, cache->stamp, C, r, K_new, V_new, ck, n_new,
              frame_id, jstar, merged, win, grp, rank, victims, hs, merge_map, cache->len, rep_mode, plan_scratch,
              (int)PS_STRIDE, stats);
    FASTAR_LAUNCH_CHECK();
#undef FASTAR_TC
    if (rep_mode == FASTAR_REP_MEAN) {
        const dim3 rgrid((n_new + 63) / 64, H);
#define FASTAR_RECODE(BF, DD, RR)                                                                                     \
    hipLaunchKernelGGL((tc_recode_kernel<BF, DD, RR>), rgrid, dim3(256), 0, s, cache->K, cache->code, C, n_new, jstar, \
                       merged, codec->R, codec->qscale, codec->shift)
        if (bf && d == 128) { if (r == 32) FASTAR_RECODE(true, 128, 32); else FASTAR_RECODE(true, 128, 64); }
        else if (bf) { if (r == 32) FASTAR_RECODE(true, 64, 32); else FASTAR_RECODE(true, 64, 64); }
        else if (d == 128) { if (r == 32) FASTAR_RECODE(false, 128, 32); else FASTAR_RECODE(false, 128, 64); }
        else { if (r == 32) FASTAR_RECODE(false, 64, 32); else FASTAR_RECODE(false, 64, 64); }
#undef FASTAR_RECODE
        FASTAR_LAUNCH_CHECK();
    }
    return FASTAR_OK;
}
