// Block-sparse attention over an 8-bit floating-point copy of the cache (E4M3 keys and values; Sec. 5.1, quantised
// search, and the appendix ablation on quantisation precision, applied to the attention itself), head dimension 128,
// blocks of 128 queries and 64 keys, and the kernel that keeps that copy up to date.
//
// Layout of the copy (per head): K8 [Cp, 128] bytes, rows as in K; V8T [Cp / 64, 128, 64] bytes, the values of every
// block of 64 slots transposed (Cp = C rounded up to a multiple of 64).  A selected key block is then two contiguous
// pieces of 8 KB, both products read their LDS operands with plain 16-byte loads (no transposing loads), and one
// matrix instruction (32x32x64, 8-bit floating-point operands) covers all 64 keys of a tile in the PV product:
//   S^T = K Q^T    A = 32 keys x 64 coordinates from LDS, B = the wavefront's 32 queries in registers (E4M3);
//                  key (32g + 16kb + 4q + e) sits in A row (8q + 4g + e) of half kb, so that a lane's 32 scores are
//                  the keys 32g .. 32g+31 in the order the next product wants them;
//   O^T = V^T P^T  A = 32 value coordinates x 64 keys from LDS, B = P rounded to E4M3, straight from the score registers;
//   l = 1^T P^T    the row sums, by the same instruction on an operand of ones: numerator and denominator see the
//                  same rounded P, so the output stays a convex combination of the stored values.
// Softmax arithmetic as in the bf16 kernels: scores start from the keys' bias (log2 of the multiplicity, -inf for
// dead slots), exponent in one fma, lazily updated reference maximum.  E4M3 spans 2^-9 .. 448, so P is kept near the
// top of that range: P = 2^6 * exp2(score - reference) with the reference at most 2 octaves behind the running
// maximum (P <= 2^8); weights more than about 15 octaves below the row maximum fall out of the format and are dropped
// (the factor 2^6 cancels in O / l and is taken out of lse).
#include <type_traits>

#include "common.hpp"

namespace fastar {

namespace f8 {

constexpr int D = 128;
constexpr int TK = 64;             // keys per tile = slots per block
constexpr int TILEB = TK * D;      // 8 KiB per tile and tensor
constexpr float LN2 = 0.6931471805599453f;
constexpr float F8_MAX = 448.0f;

typedef __attribute__((ext_vector_type(8))) int i32x8;
#define LDS_PTR8(T, p) ((__attribute__((address_space(3))) T *)(p))

// chunk (16 bytes) swizzles inside a tile, applied to the global address a lane fetches and to the LDS address it
// reads: 16 lanes of one operand read then hit 16 different 16-byte slots of a 256-byte bank line
__device__ __forceinline__ int sw_k(int row) { return ((row >> 1) & 1) | (((row >> 2) & 1) << 1) | (((row >> 5) & 1) << 2); }
__device__ __forceinline__ int sw_v(int row) { return (row >> 2) & 3; }

__device__ __forceinline__ unsigned pack_fp8x4(float a, float b, float c, float d) {
    int w = 0;
    w = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, w, false);
    w = __builtin_amdgcn_cvt_pk_fp8_f32(c, d, w, true);
    return (unsigned)w;
}
__device__ __forceinline__ float clamp_f8(float x) { return fminf(fmaxf(x, -F8_MAX), F8_MAX); }

// ---- the 8-bit copy of the cache ------------------------------------------------------------------------------
// One workgroup per (block of 64 slots, head).  A block that holds no live slot stamped >= stamp_lo is left alone;
// otherwise it is rewritten whole: live slots with the codes of the stored rows, dead slots with zero.
template <bool BF16>
__global__ __launch_bounds__(256) void kv_to_fp8_kernel(const void *__restrict__ K, const void *__restrict__ V,
                                                        const int32_t *__restrict__ stamp, const int32_t *__restrict__ len,
                                                        int C, int n_blk, int stamp_lo, uint8_t *__restrict__ K8,
                                                        uint8_t *__restrict__ V8T) {
    __shared__ __attribute__((aligned(16))) uint8_t vt[D][TK + 16];   // transposed values of the block (padded rows)
    __shared__ int dirty;
    const int blk = blockIdx.x, h = blockIdx.y;
    const int tid = threadIdx.x;
    const int L = min(len[h], C);
    if (tid == 0) dirty = 0;
    __syncthreads();
    if (tid < TK) {
        const int slot = blk * TK + tid;
        if (slot < L && stamp[(size_t)h * C + slot] >= stamp_lo) dirty = 1;
    }
    __syncthreads();
    if (!dirty) return;   // uniform
    const int j = tid >> 2, part = tid & 3;   // slot of the block, quarter of its row (32 coordinates)
    const int slot = blk * TK + j;
    const size_t Cp = (size_t)n_blk * TK;
    unsigned kw[8], vw[8];
#pragma unroll
    for (int w = 0; w < 8; ++w) kw[w] = vw[w] = 0u;
    if (slot < L) {
        float kf[32], vf[32];
        if (BF16) {
            const unsigned short *kr = (const unsigned short *)K + ((size_t)h * C + slot) * D + 32 * part;
            const unsigned short *vr = (const unsigned short *)V + ((size_t)h * C + slot) * D + 32 * part;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const u32x4 a = *(const u32x4 *)(kr + 8 * q), b = *(const u32x4 *)(vr + 8 * q);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    kf[8 * q + 2 * e] = bf16_lo(a[e]); kf[8 * q + 2 * e + 1] = bf16_hi(a[e]);
                    vf[8 * q + 2 * e] = bf16_lo(b[e]); vf[8 * q + 2 * e + 1] = bf16_hi(b[e]);
                }
            }
        } else {
            const float *kr = (const float *)K + ((size_t)h * C + slot) * D + 32 * part;
            const float *vr = (const float *)V + ((size_t)h * C + slot) * D + 32 * part;
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const f32x4 a = *(const f32x4 *)(kr + 4 * q), b = *(const f32x4 *)(vr + 4 * q);
#pragma unroll
                for (int e = 0; e < 4; ++e) { kf[4 * q + e] = a[e]; vf[4 * q + e] = b[e]; }
            }
        }
#pragma unroll
        for (int w = 0; w < 8; ++w) {
            kw[w] = pack_fp8x4(clamp_f8(kf[4 * w]), clamp_f8(kf[4 * w + 1]), clamp_f8(kf[4 * w + 2]), clamp_f8(kf[4 * w + 3]));
            vw[w] = pack_fp8x4(clamp_f8(vf[4 * w]), clamp_f8(vf[4 * w + 1]), clamp_f8(vf[4 * w + 2]), clamp_f8(vf[4 * w + 3]));
        }
    }
    {
        uint8_t *dst = K8 + ((size_t)h * Cp + slot) * D + 32 * part;
        u32x4 lo = {kw[0], kw[1], kw[2], kw[3]}, hi = {kw[4], kw[5], kw[6], kw[7]};
        *(u32x4 *)dst = lo;
        *(u32x4 *)(dst + 16) = hi;
    }
#pragma unroll
    for (int w = 0; w < 8; ++w)
#pragma unroll
        for (int b = 0; b < 4; ++b) vt[32 * part + 4 * w + b][j] = (uint8_t)(vw[w] >> (8 * b));
    __syncthreads();
    {
        // 128 rows of 64 bytes: thread -> row tid/2, half tid%2 (32 bytes)
        const int row = tid >> 1, half = tid & 1;
        uint8_t *dst = V8T + (((size_t)h * n_blk + blk) * D + row) * TK + 32 * half;
        *(u32x4 *)dst = *(const u32x4 *)(&vt[row][32 * half]);
        *(u32x4 *)(dst + 16) = *(const u32x4 *)(&vt[row][32 * half + 16]);
    }
}

// ---- attention ------------------------------------------------------------------------------------------------
struct __attribute__((aligned(16))) TileMeta {
    float bias[TK];  // log2(cnt) of the tile's keys in units of raw scores (divided by scale * log2 e), -inf when dead
    int blk;         // block to load (a masked tile loads block 0, which is live)
    int pad[3];
};

constexpr int OSTR = D + 8;                                   // bf16 elements per staged output row
constexpr int STAGE_BYTES = 4 * TILEB;                        // K and V, two stages each
constexpr int OUT_BYTES = 4 * 32 * OSTR * 2;                  // output staging of the four wavefronts
constexpr int META_OFF = OUT_BYTES > STAGE_BYTES ? OUT_BYTES : STAGE_BYTES;
constexpr int LDS_BYTES = META_OFF + 3 * (int)sizeof(TileMeta);

__device__ __forceinline__ i32x8 lds_read_32(const unsigned char *p0, const unsigned char *p1) {
    const i32x4 lo = *(const i32x4 *)p0, hi = *(const i32x4 *)p1;
    i32x8 r = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return r;
}
__device__ __forceinline__ f32x16 mfma_f8(i32x8 a, i32x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 0, 0, 0, 0, 0, 0);   // both operands E4M3, no scales
}

// Query block b of head h over the entries t_begin <= t < t_end of its list (one entry = one tile).  part == nullptr:
// normalised output rows and lse are written (the range must then be the whole list).  part != nullptr: the unnormalised
// O^T accumulators ([wave][32-row block of d][register][lane]), then the reference maxima and the row sums
// ([wave][lane] each): the fragment layout that the combination launch of the split bf16 kernel reads.
// All 256 threads of a workgroup; may be called again by the same workgroup for another block.
__device__ __forceinline__ void attend_item_fp8(
    const unsigned short *__restrict__ Q, const uint8_t *__restrict__ K8, const uint8_t *__restrict__ V8T,
    const int32_t *__restrict__ cnt, const int32_t *__restrict__ len, const int32_t *__restrict__ sel,
    const int32_t *__restrict__ nsel, int n_q, int C, int n_blk, int n_sel, int n_qb, float scale_log2,
    float inv_scale_log2, unsigned short *__restrict__ O, float *__restrict__ lse, unsigned char *lds, int h, int b,
    int t_begin, int t_end, float *__restrict__ part) {
    unsigned char *kbuf = lds;
    unsigned char *vbuf = lds + 2 * TILEB;
    TileMeta *meta = (TileMeta *)(lds + META_OFF);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, g = lane >> 5;
    const int L = min(len[h], C);
    const int n_live_blk = (L + TK - 1) / TK;
    const int nt_all = L > 0 ? min(nsel[(size_t)h * n_qb + b], n_sel) : 0;   // one selection entry = one tile
    const int nt = max(0, min(nt_all, t_end) - t_begin);                     // tiles of this call: entries t_begin .. t_begin + nt - 1
    const int32_t *sel_row = sel + ((size_t)h * n_qb + b) * n_sel + t_begin;
    const int32_t *cnt_h = cnt ? cnt + (size_t)h * C : nullptr;
    const uint8_t *Kh = K8 + (size_t)h * n_blk * TK * D;
    const uint8_t *Vh = V8T + (size_t)h * n_blk * TILEB;

    // queries of this wavefront as the B operand of the score product: lane (query col, half g) holds coordinates
    // 64s + 32g .. +31 of k-step s, rounded to E4M3
    const int q_idx = b * 128 + wave * 32 + col;
    i32x8 qf[2];
    {
        const unsigned short *qrow = Q + ((size_t)h * n_q + min(q_idx, n_q - 1)) * D;
#pragma unroll
        for (int s = 0; s < 2; ++s) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const u32x4 w = *(const u32x4 *)(qrow + 64 * s + 32 * g + 8 * q);
                qf[s][2 * q] = (int)pack_fp8x4(clamp_f8(bf16_lo(w[0])), clamp_f8(bf16_hi(w[0])), clamp_f8(bf16_lo(w[1])),
                                               clamp_f8(bf16_hi(w[1])));
                qf[s][2 * q + 1] = (int)pack_fp8x4(clamp_f8(bf16_lo(w[2])), clamp_f8(bf16_hi(w[2])), clamp_f8(bf16_lo(w[3])),
                                                   clamp_f8(bf16_hi(w[3])));
            }
        }
    }
    f32x16 o_acc[D / 32], l_acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        l_acc[v] = 0.0f;
#pragma unroll
        for (int db = 0; db < D / 32; ++db) o_acc[db][v] = 0.0f;
    }
    i32x8 ones;
#pragma unroll
    for (int w = 0; w < 8; ++w) ones[w] = 0x38383838;   // 1.0 in every byte
    float m_ref = -INFINITY, neg_ms = 0.0f;
    constexpr float P_OFF = 6.0f;                  // P = 2^P_OFF * exp2(score - reference)
    const float tau_raw = 2.0f * inv_scale_log2;   // the reference may lag the true maximum by 2 octaves: P <= 2^8

    // direct global -> LDS loads of one tile: eight 1-KiB instructions per tensor, two per wavefront
    auto issue_loads = [&](int blk, int stage) {
        const uint8_t *kt = Kh + (size_t)blk * TILEB;
        const uint8_t *vt = Vh + (size_t)blk * TILEB;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int inst = 2 * wave + i;
            const int krow = 8 * inst + (lane >> 3), kpos = lane & 7;
            const int vrow = 16 * inst + (lane >> 2), vpos = lane & 3;
            const uint8_t *ksrc = kt + krow * D + ((kpos ^ sw_k(krow)) << 4);
            const uint8_t *vsrc = vt + vrow * TK + ((vpos ^ sw_v(vrow)) << 4);
            __builtin_amdgcn_global_load_lds(ksrc, LDS_PTR8(unsigned, kbuf + stage * TILEB + inst * 1024), 16, 0, 0);
            __builtin_amdgcn_global_load_lds(vsrc, LDS_PTR8(unsigned, vbuf + stage * TILEB + inst * 1024), 16, 0, 0);
        }
    };
    // tile bookkeeping, two tiles ahead, by the first 64 threads (one per key of the tile)
    auto sel_entry = [&](int tile) -> int { return (tid < TK && tile < nt) ? sel_row[tile] : -1; };
    auto fill_meta = [&](TileMeta &m, int kb, int cnt_v) {
        if (tid < TK) {
            const bool blk_ok = kb >= 0 && kb < n_live_blk;
            const int key = kb * TK + tid;
            const bool live = blk_ok && key < L;
            m.bias[tid] = live ? (cnt_h ? __log2f((float)cnt_v) * inv_scale_log2 : 0.0f) : -INFINITY;
            if (tid == 0) m.blk = blk_ok ? kb : 0;
        }
    };
    auto cnt_of = [&](int kb) -> int {
        const int key = kb * TK + tid;
        return (tid < TK && cnt_h && kb >= 0 && key < L) ? cnt_h[key] : 1;
    };
    int kb_ahead = -1;
    if (nt > 0) {
        const int kb0 = sel_entry(0), kb1 = sel_entry(1);
        fill_meta(meta[0], kb0, cnt_of(kb0));
        if (nt > 1) fill_meta(meta[1], kb1, cnt_of(kb1));
        if (nt > 2) kb_ahead = sel_entry(2);
        __syncthreads();
        issue_loads(meta[0].blk, 0);
    }
    // per-lane LDS offsets of the operand reads (tile-independent)
    unsigned koff[2][2];   // [key half kb][k-step s]: first of the two chunks; the second is that offset ^ 16
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
        const int row = 32 * ((col >> 2) & 1) + 16 * kb + 4 * (col >> 3) + (col & 3);
#pragma unroll
        for (int s = 0; s < 2; ++s) koff[kb][s] = row * D + (((4 * s + 2 * g) ^ sw_k(row)) << 4);
    }
    unsigned voff[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db) {
        const int row = 32 * db + col;
        voff[db] = row * TK + (((2 * g) ^ sw_v(row)) << 4);
    }

    auto tile_step = [&](int t, auto stage_c) {
        constexpr int STAGE = decltype(stage_c)::value;
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wavefront's share of tile t has landed
        __syncthreads();                     // ... and everyone else's; tile t-1 fully consumed
        int cnt2 = 1, kb3 = -1;
        const int kb2 = kb_ahead;
        if (t + 2 < nt) {
            cnt2 = cnt_of(kb2);
            if (t + 3 < nt) kb3 = sel_entry(t + 3);
        }
        if (t + 1 < nt) issue_loads(meta[(t + 1) % 3].blk, STAGE ^ 1);
        const TileMeta &mt = meta[t % 3];
        const unsigned char *ks = kbuf + STAGE * TILEB, *vs = vbuf + STAGE * TILEB;
        // scores start from the keys' bias: register 4q+e of half kb is key 32g + 16kb + 4q + e
        f32x16 s_acc[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const f32x4 bv = *(const f32x4 *)(&mt.bias[32 * g + 16 * kb + 4 * q4]);
#pragma unroll
                for (int e = 0; e < 4; ++e) s_acc[kb][4 * q4 + e] = bv[e];
            }
        i32x8 ka[2][2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int s = 0; s < 2; ++s) ka[kb][s] = lds_read_32(ks + koff[kb][s], ks + (koff[kb][s] ^ 16u));
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int s = 0; s < 2; ++s) s_acc[kb] = mfma_f8(ka[kb][s], qf[s], s_acc[kb]);
        // V^T operands: issued now, they land during the softmax arithmetic
        i32x8 va[D / 32];
#pragma unroll
        for (int db = 0; db < D / 32; ++db) va[db] = lds_read_32(vs + voff[db], vs + (voff[db] ^ 16u));
        float mx = s_acc[0][0];
#pragma unroll
        for (int v = 1; v < 16; ++v) mx = fmaxf(mx, s_acc[0][v]);
#pragma unroll
        for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s_acc[1][v]);
        mx = fmaxf(mx, shfl_xor(mx, 32));
        if (__any(mx > m_ref + tau_raw)) {   // wave-uniform
            const float m_new = fmaxf(m_ref, mx);
            const float alpha = m_ref == -INFINITY ? 0.0f : __builtin_amdgcn_exp2f((m_ref - m_new) * scale_log2);
            m_ref = m_new;
            neg_ms = m_new == -INFINITY ? 0.0f : P_OFF - m_new * scale_log2;
            l_acc[0] *= alpha;
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) o_acc[db][v] *= alpha;
        }
        i32x8 pf;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                float p[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) p[e] = __builtin_amdgcn_exp2f(fmaf(s_acc[kb][4 * q4 + e], scale_log2, neg_ms));
                pf[4 * kb + q4] = (int)pack_fp8x4(p[0], p[1], p[2], p[3]);
            }
        l_acc = mfma_f8(ones, pf, l_acc);
#pragma unroll
        for (int db = 0; db < D / 32; ++db) o_acc[db] = mfma_f8(va[db], pf, o_acc[db]);
        // bookkeeping of tile t+2
        if (t + 2 < nt) fill_meta(meta[(t + 2) % 3], kb2, cnt2);
        kb_ahead = kb3;
    };
    for (int t = 0; t < nt; t += 2) {
        tile_step(t, std::integral_constant<int, 0>{});
        if (t + 1 < nt) tile_step(t + 1, std::integral_constant<int, 1>{});
    }

    const float l_tot = l_acc[0];
    if (part) {   // a fragment: the combination launch normalises
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) part[((wave * (D / 32) + db) * 16 + v) * 64 + lane] = o_acc[db][v];
        part[4 * ATTN_PART_O_FLOATS + wave * 64 + lane] = m_ref;
        part[4 * ATTN_PART_O_FLOATS + 4 * 64 + wave * 64 + lane] = l_tot;
        __syncthreads();   // the tile stages and the bookkeeping are free for the next block
        return;
    }
    // epilogue: normalise, transpose through LDS, store rows coalesced
    const float inv = l_tot > 0.0f ? 1.0f / l_tot : 0.0f;
    __syncthreads();
    unsigned short *Os = (unsigned short *)lds + (size_t)wave * 32 * OSTR;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
            bf16x4 w;
#pragma unroll
            for (int e = 0; e < 4; ++e) w[e] = (__bf16)(o_acc[db][4 * q4 + e] * inv);
            *(bf16x4 *)(Os + col * OSTR + 32 * db + 8 * q4 + 4 * g) = w;
        }
    __syncthreads();
    {
        const int rr = lane >> 4, cc = lane & 15;
#pragma unroll
        for (int it = 0; it < 8; ++it) {
            const int r = it * 4 + rr;
            const int qi = b * 128 + wave * 32 + r;
            if (qi < n_q) *(u32x4 *)(O + ((size_t)h * n_q + qi) * D + cc * 8) = *(const u32x4 *)(Os + r * OSTR + cc * 8);
        }
    }
    if (lse && g == 0 && q_idx < n_q)
        lse[(size_t)h * n_q + q_idx] = l_tot > 0.0f ? (m_ref * scale_log2 - 6.0f + __log2f(l_tot)) * LN2 : -INFINITY;
    __syncthreads();   // the staged output rows have been read: the tile stages are free for the next block
}

// One query block per workgroup; two workgroups per CU, started as slots free up.
__global__ __launch_bounds__(256, 2) void attn_fp8_d128_kernel(
    const unsigned short *__restrict__ Q, const uint8_t *__restrict__ K8, const uint8_t *__restrict__ V8T,
    const int32_t *__restrict__ cnt, const int32_t *__restrict__ len, const int32_t *__restrict__ sel,
    const int32_t *__restrict__ nsel, int n_q, int C, int n_blk, int n_sel, int n_qb, int H, float scale_log2,
    float inv_scale_log2, unsigned short *__restrict__ O, float *__restrict__ lse) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    // workgroup -> (head, query block): each XCD gets a contiguous range of (head, block) pairs
    const int total = n_qb * H;
    const int wg = blockIdx.x;
    const int per = (total + 7) / 8;
    const int item = (wg & 7) * per + (wg >> 3);
    if (item >= total) return;
    attend_item_fp8(Q, K8, V8T, cnt, len, sel, nsel, n_q, C, n_blk, n_sel, n_qb, scale_log2, inv_scale_log2, O, lse, lds,
                    item / n_qb, item % n_qb, 0, INT_MAX, nullptr);
}

// The split launch (see the bf16 kernel of the same structure in attention_d128.hip): the first n_plain workgroups take one
// whole query block each, in the plain kernel's order; the others take equal shares of the tiles of the blocks left over.
__global__ __launch_bounds__(256, 2) void attn_fp8_d128_sk_kernel(
    const unsigned short *__restrict__ Q, const uint8_t *__restrict__ K8, const uint8_t *__restrict__ V8T,
    const int32_t *__restrict__ cnt, const int32_t *__restrict__ len, const int32_t *__restrict__ sel,
    const int32_t *__restrict__ nsel, int n_q, int C, int n_blk, int n_sel, int n_qb, TailMap tm, int n_plain, int NT,
    float scale_log2, float inv_scale_log2, unsigned short *__restrict__ O, float *__restrict__ lse, float *__restrict__ ws) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    const int P = (int)gridDim.x - n_plain;                        // a multiple of 8
    const int wg = (int)blockIdx.x - n_plain;
    const int i = (wg & 7) * (P >> 3) + (wg >> 3);                 // neighbouring shares on one XCD: those of its own range
    const int direct = wg < 0 ? ((int)blockIdx.x & 7) * tm.per + ((int)blockIdx.x >> 3) : -1;
    const long long W = tm.tiles(NT);
    long long v = wg < 0 ? 0 : i * W / P;
    const long long v_end = wg < 0 ? NT : (i + 1) * W / P;
    while (v < v_end) {
        const int vi = (int)(v / NT);
        const int t_begin = (int)(v - (long long)vi * NT);
        const int t_end = (int)min((long long)NT, v_end - (long long)vi * NT);
        const int item = direct >= 0 ? direct : tm.item(vi);
        if (item < tm.total) {   // uniform over the workgroup
            float *part = nullptr;
            if (t_begin > 0 || t_end < NT) part = ws + ((size_t)i * 2 + (t_begin > 0 ? 0 : 1)) * ATTN_PART_FLOATS;
            attend_item_fp8(Q, K8, V8T, cnt, len, sel, nsel, n_q, C, n_blk, n_sel, n_qb, scale_log2, inv_scale_log2, O, lse,
                            lds, item / n_qb, item % n_qb, t_begin, t_end, part);
        }
        v = (long long)vi * NT + t_end;
    }
}

}  // namespace f8

int attn_fp8_setup() {
    static DeviceOnce once;
    return once.run([](int) {
        return hipFuncSetAttribute((const void *)f8::attn_fp8_d128_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                   f8::LDS_BYTES) == hipSuccess &&
                       hipFuncSetAttribute((const void *)f8::attn_fp8_d128_sk_kernel,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, f8::LDS_BYTES) == hipSuccess
                   ? FASTAR_OK
                   : FASTAR_ERR_HIP;
    });
}

}  // namespace fastar

using namespace fastar;

extern "C" int fastar_kv_to_fp8(const fastar_cache *cache, int32_t stamp_lo, uint8_t *K8, uint8_t *V8T, void *stream) {
    if (!cache || !K8 || !V8T) return FASTAR_ERR_INVALID_ARG;
    if (!cache->K || !cache->V || !cache->stamp || !cache->len) return FASTAR_ERR_INVALID_ARG;
    const int H = cache->H, C = cache->C;
    if (H <= 0 || C <= 0) return FASTAR_ERR_INVALID_ARG;
    if (cache->dtype != FASTAR_F32 && cache->dtype != FASTAR_BF16) return FASTAR_ERR_INVALID_ARG;
    if (cache->d != 128) return FASTAR_ERR_UNSUPPORTED;
    if (((uintptr_t)cache->K & 15) || ((uintptr_t)cache->V & 15) || ((uintptr_t)K8 & 15) || ((uintptr_t)V8T & 15))
        return FASTAR_ERR_INVALID_ARG;
    const int n_blk = (C + f8::TK - 1) / f8::TK;
    const dim3 grid(n_blk, H);
    if (cache->dtype == FASTAR_BF16)
        hipLaunchKernelGGL(f8::kv_to_fp8_kernel<true>, grid, dim3(256), 0, (hipStream_t)stream, cache->K, cache->V,
                           cache->stamp, cache->len, C, n_blk, stamp_lo, K8, V8T);
    else
        hipLaunchKernelGGL(f8::kv_to_fp8_kernel<false>, grid, dim3(256), 0, (hipStream_t)stream, cache->K, cache->V,
                           cache->stamp, cache->len, C, n_blk, stamp_lo, K8, V8T);
    FASTAR_LAUNCH_CHECK();
    return FASTAR_OK;
}

static int sparse_attn_fp8_impl(const void *Q, int n_q, const uint8_t *K8, const uint8_t *V8T, const int32_t *cnt,
                                const int32_t *len, int H, int C, int d, const int32_t *sel, const int32_t *nsel, int BQ,
                                int BK, int n_sel, float scale, void *O, float *lse, void *ws, void *stream);

extern "C" int sparse_attn_fwd_fp8(const void *Q, int n_q, const uint8_t *K8, const uint8_t *V8T, const int32_t *cnt,
                                   const int32_t *len, int H, int C, int d, const int32_t *sel, const int32_t *nsel,
                                   int BQ, int BK, int n_sel, float scale, void *O, float *lse, void *stream) {
    return sparse_attn_fp8_impl(Q, n_q, K8, V8T, cnt, len, H, C, d, sel, nsel, BQ, BK, n_sel, scale, O, lse, nullptr, stream);
}

extern "C" int sparse_attn_fwd_fp8_ws(const void *Q, int n_q, const uint8_t *K8, const uint8_t *V8T, const int32_t *cnt,
                                      const int32_t *len, int H, int C, int d, const int32_t *sel, const int32_t *nsel,
                                      int BQ, int BK, int n_sel, float scale, void *O, float *lse, void *ws,
                                      size_t ws_bytes, void *stream) {
    if (!ws || ((uintptr_t)ws & 255)) return FASTAR_ERR_INVALID_ARG;
    if (ws_bytes < (size_t)ATTN_SHARE_WORKGROUPS * 2 * ATTN_PART_FLOATS * sizeof(float)) return FASTAR_ERR_WORKSPACE;
    return sparse_attn_fp8_impl(Q, n_q, K8, V8T, cnt, len, H, C, d, sel, nsel, BQ, BK, n_sel, scale, O, lse, ws, stream);
}

static int sparse_attn_fp8_impl(const void *Q, int n_q, const uint8_t *K8, const uint8_t *V8T, const int32_t *cnt,
                                const int32_t *len, int H, int C, int d, const int32_t *sel, const int32_t *nsel, int BQ,
                                int BK, int n_sel, float scale, void *O, float *lse, void *ws, void *stream) {
    if (!Q || !K8 || !V8T || !len || !sel || !nsel || !O) return FASTAR_ERR_INVALID_ARG;
    if (H <= 0 || n_q <= 0 || C <= 0 || n_sel <= 0) return FASTAR_ERR_INVALID_ARG;
    if (!(scale > 0.0f) || !(scale < INFINITY)) return FASTAR_ERR_INVALID_ARG;
    if (((uintptr_t)Q & 15) || ((uintptr_t)K8 & 15) || ((uintptr_t)V8T & 15) || ((uintptr_t)O & 15))
        return FASTAR_ERR_INVALID_ARG;
    if (d != 128 || BQ != 128 || BK != 64) return FASTAR_ERR_UNSUPPORTED;
    if (const int rc = attn_fp8_setup(); rc != FASTAR_OK) return rc;
    const int n_qb = (n_q + 127) / 128;
    const int n_blk = (C + f8::TK - 1) / f8::TK;
    const float scale_log2 = scale * 1.4426950408889634f;
    // with a workspace, a launch that would end in a short last round of workgroups is split (one entry = one tile)
    const int full_per = ws ? attn_split_full_per(n_qb * H, n_sel) : 0;
    if (full_per > 0) {
        const TailMap tm = {(n_qb * H + 7) / 8, full_per, n_qb * H};
        const int n_plain = 8 * full_per;
        hipLaunchKernelGGL(f8::attn_fp8_d128_sk_kernel, dim3(n_plain + ATTN_SHARE_WORKGROUPS), dim3(256), f8::LDS_BYTES,
                           (hipStream_t)stream, (const unsigned short *)Q, K8, V8T, cnt, len, sel, nsel, n_q, C, n_blk,
                           n_sel, n_qb, tm, n_plain, n_sel, scale_log2, 1.0f / scale_log2, (unsigned short *)O, lse,
                           (float *)ws);
        FASTAR_LAUNCH_CHECK();
        return launch_attn_combine(ws, n_q, n_qb, tm, n_sel, scale_log2, -6.0f, O, lse, (hipStream_t)stream);
    }
    const dim3 grid((unsigned)(((n_qb * H + 7) / 8) * 8));
    hipLaunchKernelGGL(f8::attn_fp8_d128_kernel, grid, dim3(256), f8::LDS_BYTES, (hipStream_t)stream,
                       (const unsigned short *)Q, K8, V8T, cnt, len, sel, nsel, n_q, C, n_blk, n_sel, n_qb, H, scale_log2,
                       1.0f / scale_log2, (unsigned short *)O, lse);
    FASTAR_LAUNCH_CHECK();
    return FASTAR_OK;
}
