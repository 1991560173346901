// Block-sparse attention over the selected key blocks (Eq. 1 restricted to the candidate set of
// Sec. 5.1; logits shifted by +ln(cnt) as Lemma 1 prescribes for merged groups).
//
// bf16 path (matrix cores).  One workgroup = one query block of BQ = 32*NW queries, one wavefront
// = 32 queries.  Key tiles of 64 rows are gathered by the selection list into LDS (K row-major,
// V transposed so that a lane can fetch 4 consecutive keys of one value column), the next tile is
// prefetched into registers while the current one is consumed.  Both contractions are computed
// "transposed" so that every per-query quantity lives in one lane:
//     S^T = K Q^T   (A = K tile from LDS, B = Q fragment held in registers)  -> lane = query, regs = keys
//     O^T = V^T P^T (A = V^T tile from LDS, B = P^T = the S^T registers, no data movement) -> lane = query
// Softmax runs in fp32 in the log2 domain with a running maximum; masked keys (padding of the list,
// slots beyond len) get a -inf bias and zeroed K/V rows.
//
// fp32 path (small reference-precision case): one thread per query, K/V tiles broadcast from LDS.
#include "common.hpp"

namespace fastar {

constexpr int TK = 64;  // keys per tile
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

struct __attribute__((aligned(16))) TileMeta {
    int idx[TK];     // cache row of each tile position, -1 = masked
    float bias[TK];  // log2(cnt) of that row, -inf when masked
};

// Fill the row table of tile `t` (threads 0..63 of the workgroup).
__device__ __forceinline__ void fill_meta(TileMeta &m, int t, const int32_t *__restrict__ sel_row, int n_listed,
                                          int bk_shift, int L, const int32_t *__restrict__ cnt_h) {
    const int p = threadIdx.x;
    if (p < TK) {
        const int listpos = t * TK + p;
        const int entry = listpos >> bk_shift;
        int key = -1;
        if (entry < n_listed) {
            const int kb = sel_row[entry];
            if (kb >= 0) {
                key = (kb << bk_shift) + (listpos & ((1 << bk_shift) - 1));
                if (key >= L) key = -1;
            }
        }
        float bias = -INFINITY;
        if (key >= 0) bias = cnt_h ? __log2f((float)cnt_h[key]) : 0.0f;
        m.idx[p] = key;
        m.bias[p] = bias;
    }
}

template <int D, int NW>
struct AttnCfg {
    static constexpr int NT = NW * 64;
    static constexpr int KSTR = D + 8;    // bf16 elements per K row in LDS (16-byte pad: conflict-free b128 reads)
    static constexpr int VSTR = TK + 4;   // bf16 elements per V^T row in LDS
    static constexpr int CPR = D / 8;     // 16-byte chunks per row
    static constexpr int KCH = TK * CPR / NT;                  // K chunks staged per thread
    static constexpr int VBLK_TOTAL = (TK / 4) * CPR;          // 4-key x 8-column blocks per tile
    static constexpr int VBLK = (VBLK_TOTAL + NT - 1) / NT;    // per thread
    static constexpr int K_BYTES = TK * KSTR * 2;
    static constexpr int V_BYTES = D * VSTR * 2;
    static constexpr int O_BYTES = NW * 32 * KSTR * 2;         // epilogue staging, reuses the tile space
    static constexpr int TILE_BYTES = (K_BYTES + V_BYTES) > O_BYTES ? (K_BYTES + V_BYTES) : O_BYTES;
};

template <int D, int NW>
__global__ __launch_bounds__(NW * 64, 2) void attn_bf16_kernel(
    const unsigned short *__restrict__ Q, const unsigned short *__restrict__ K, const unsigned short *__restrict__ V,
    const int32_t *__restrict__ cnt, const int32_t *__restrict__ len, const int32_t *__restrict__ sel,
    const int32_t *__restrict__ nsel, int n_q, int C, int bk_shift, int n_sel, int n_qb, int H, float scale_log2,
    unsigned short *__restrict__ O, float *__restrict__ lse) {
    typedef AttnCfg<D, NW> Cfg;
    constexpr int NT = Cfg::NT, KSTR = Cfg::KSTR, VSTR = Cfg::VSTR, CPR = Cfg::CPR;
    __shared__ __attribute__((aligned(16))) unsigned char tile_mem[Cfg::TILE_BYTES];
    __shared__ TileMeta meta[3];
    unsigned short *Ks = (unsigned short *)tile_mem;
    unsigned short *Vt = (unsigned short *)(tile_mem + Cfg::K_BYTES);

    // workgroup -> (head, query block).  Workgroups are dealt round-robin to the 8 XCDs; give each
    // XCD a contiguous range of (head, block) pairs so that the K/V of a head stay in one L2.
    int h, b;
    {
        const int total = n_qb * H;
        const int wg = blockIdx.x;
        const int per = (total + 7) / 8;      // the grid holds 8 * per workgroups
        const int item = (wg & 7) * per + (wg >> 3);
        if (item >= total) return;            // padding of the last XCD's range (uniform)
        h = item / n_qb;
        b = item % n_qb;
    }
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, g = lane >> 5;
    const int L = min(len[h], C);
    const int n_listed = min(nsel[(size_t)h * n_qb + b], n_sel);
    const int32_t *sel_row = sel + ((size_t)h * n_qb + b) * n_sel;
    const int32_t *cnt_h = cnt ? cnt + (size_t)h * C : nullptr;
    const unsigned short *Kh = K + (size_t)h * C * D;
    const unsigned short *Vh = V + (size_t)h * C * D;
    const int nt = ((n_listed << bk_shift) + TK - 1) / TK;

    // Q fragments of this wavefront's 32 queries (B operand: column = query, k-slots = 8 coordinates)
    const int q_idx = b * (NW * 32) + wave * 32 + col;
    bf16x8 qf[D / 16];
    {
        const unsigned short *qrow = Q + ((size_t)h * n_q + min(q_idx, n_q - 1)) * D;
#pragma unroll
        for (int s = 0; s < D / 16; ++s) qf[s] = *(const bf16x8 *)(qrow + 16 * s + 8 * g);
    }

    f32x16 o_acc[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) o_acc[db][v] = 0.0f;
    float m_run = -INFINITY, l_run = 0.0f;

    u32x4 kst[Cfg::KCH];
    u32x4 vst[Cfg::VBLK][4];
    auto issue_loads = [&](const TileMeta &m) {
#pragma unroll
        for (int c = 0; c < Cfg::KCH; ++c) {
            const int ch = tid + c * NT;
            const int row = ch / CPR, cc = ch % CPR;
            const int key = m.idx[row];
            u32x4 z = {0, 0, 0, 0};
            kst[c] = key >= 0 ? *(const u32x4 *)(Kh + (size_t)key * D + cc * 8) : z;
        }
#pragma unroll
        for (int vb = 0; vb < Cfg::VBLK; ++vb) {
            const int blk = tid + vb * NT;
            const int a = blk / CPR, cc = blk % CPR;
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                u32x4 z = {0, 0, 0, 0};
                int key = -1;
                if (blk < Cfg::VBLK_TOTAL) key = m.idx[4 * a + rr];
                vst[vb][rr] = key >= 0 ? *(const u32x4 *)(Vh + (size_t)key * D + cc * 8) : z;
            }
        }
    };
    auto store_tiles = [&]() {
#pragma unroll
        for (int c = 0; c < Cfg::KCH; ++c) {
            const int ch = tid + c * NT;
            const int row = ch / CPR, cc = ch % CPR;
            *(u32x4 *)(Ks + row * KSTR + cc * 8) = kst[c];
        }
#pragma unroll
        for (int vb = 0; vb < Cfg::VBLK; ++vb) {
            const int blk = tid + vb * NT;
            if (blk < Cfg::VBLK_TOTAL) {
                const int a = blk / CPR, cc = blk % CPR;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const unsigned w0 = vst[vb][0][q], w1 = vst[vb][1][q], w2 = vst[vb][2][q], w3 = vst[vb][3][q];
                    u32x2 even = {(w0 & 0xFFFFu) | (w1 << 16), (w2 & 0xFFFFu) | (w3 << 16)};
                    u32x2 odd = {(w0 >> 16) | (w1 & 0xFFFF0000u), (w2 >> 16) | (w3 & 0xFFFF0000u)};
                    *(u32x2 *)(Vt + (cc * 8 + 2 * q) * VSTR + 4 * a) = even;
                    *(u32x2 *)(Vt + (cc * 8 + 2 * q + 1) * VSTR + 4 * a) = odd;
                }
            }
        }
    };

    if (nt > 0) {
        fill_meta(meta[0], 0, sel_row, n_listed, bk_shift, L, cnt_h);
        if (nt > 1) fill_meta(meta[1], 1, sel_row, n_listed, bk_shift, L, cnt_h);
        __syncthreads();
        issue_loads(meta[0]);
    }
    for (int t = 0; t < nt; ++t) {
        __syncthreads();  // tile t-1 fully consumed; row table of tile t+1 visible
        store_tiles();
        __syncthreads();
        if (t + 1 < nt) issue_loads(meta[(t + 1) % 3]);
        if (t + 2 < nt) fill_meta(meta[(t + 2) % 3], t + 2, sel_row, n_listed, bk_shift, L, cnt_h);
        const TileMeta &mt = meta[t % 3];

        // S^T = K Q^T : two blocks of 32 keys x 32 queries
        f32x16 s_acc[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int v = 0; v < 16; ++v) s_acc[kb][v] = 0.0f;
#pragma unroll
            for (int s = 0; s < D / 16; ++s) {
                const bf16x8 a = *(const bf16x8 *)(Ks + (32 * kb + col) * KSTR + 16 * s + 8 * g);
                s_acc[kb] = mfma_bf16_32x32x16(a, qf[s], s_acc[kb]);
            }
        }
        // logits in the log2 domain, masked keys at -inf
        float mx = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const f32x4 bv = *(const f32x4 *)(&mt.bias[32 * kb + 8 * q4 + 4 * g]);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float sv = fmaf(s_acc[kb][4 * q4 + e], scale_log2, bv[e]);
                    s_acc[kb][4 * q4 + e] = sv;
                    mx = fmaxf(mx, sv);
                }
            }
        mx = fmaxf(mx, shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);
        const float m_safe = m_new == -INFINITY ? 0.0f : m_new;
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_safe);
        float psum = 0.0f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const float p = __builtin_amdgcn_exp2f(s_acc[kb][v] - m_safe);
                s_acc[kb][v] = p;
                psum += p;
            }
        l_run = l_run * alpha + psum;
        m_run = m_new;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) o_acc[db][v] *= alpha;

        // O^T += V^T P^T : four steps of 16 keys
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                bf16x8 pf;
#pragma unroll
                for (int e = 0; e < 8; ++e) pf[e] = (__bf16)s_acc[kb][8 * half + e];
                const int kbase = 32 * kb + 16 * half;
#pragma unroll
                for (int db = 0; db < D / 32; ++db) {
                    const unsigned short *vp = Vt + (32 * db + col) * VSTR + kbase + 4 * g;
                    const u32x2 lo = *(const u32x2 *)vp;
                    const u32x2 hi = *(const u32x2 *)(vp + 8);
                    u32x4 w = {lo[0], lo[1], hi[0], hi[1]};
                    bf16x8 a;
                    __builtin_memcpy(&a, &w, 16);
                    o_acc[db] = mfma_bf16_32x32x16(a, pf, o_acc[db]);
                }
            }
    }

    // epilogue: normalise, transpose through LDS, store rows coalesced
    const float l_tot = l_run + shfl_xor(l_run, 32);
    const float inv = l_tot > 0.0f ? 1.0f / l_tot : 0.0f;
    __syncthreads();
    unsigned short *Os = (unsigned short *)tile_mem + (size_t)wave * 32 * KSTR;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            u32x2 w = {pack_bf16x2(o_acc[db][4 * q4] * inv, o_acc[db][4 * q4 + 1] * inv),
                       pack_bf16x2(o_acc[db][4 * q4 + 2] * inv, o_acc[db][4 * q4 + 3] * inv)};
            *(u32x2 *)(Os + col * KSTR + 32 * db + 8 * q4 + 4 * g) = w;
        }
    __syncthreads();
    {
        constexpr int LPR = CPR;          // lanes per row (16-byte chunks)
        constexpr int RPI = 64 / LPR;     // rows per iteration
        const int rr = lane / LPR, cc = lane % LPR;
#pragma unroll
        for (int it = 0; it < 32 / RPI; ++it) {
            const int r = it * RPI + rr;
            const int qi = b * (NW * 32) + wave * 32 + r;
            if (qi < n_q) *(u32x4 *)(O + ((size_t)h * n_q + qi) * D + cc * 8) = *(const u32x4 *)(Os + r * KSTR + cc * 8);
        }
    }
    if (lse && g == 0 && q_idx < n_q)
        lse[(size_t)h * n_q + q_idx] = l_tot > 0.0f ? (m_run + __log2f(l_tot)) * LN2 : -INFINITY;
}

// ---- fp32 reference-precision path ----------------------------------------------------------------------
constexpr int TKF = 32;  // keys per LDS sub-tile of the fp32 path

template <int D>
__global__ __launch_bounds__(128) void attn_f32_kernel(const float *__restrict__ Q, const float *__restrict__ K,
                                                       const float *__restrict__ V, const int32_t *__restrict__ cnt,
                                                       const int32_t *__restrict__ len, const int32_t *__restrict__ sel,
                                                       const int32_t *__restrict__ nsel, int n_q, int C, int BQ, int BK,
                                                       int n_sel, int n_qb, float scale_log2, float *__restrict__ O,
                                                       float *__restrict__ lse) {
    __shared__ __attribute__((aligned(16))) float Ks[TKF * D];
    __shared__ __attribute__((aligned(16))) float Vs[TKF * D];
    __shared__ float bias[TKF];
    const int b = blockIdx.x, h = blockIdx.y, tid = threadIdx.x;
    const int L = min(len[h], C);
    const int n_listed = min(nsel[(size_t)h * n_qb + b], n_sel);
    const int32_t *sel_row = sel + ((size_t)h * n_qb + b) * n_sel;
    const int qi = b * BQ + tid;
    const bool active = tid < BQ && qi < n_q;
    float q[D], o[D];
    {
        const float *qrow = Q + ((size_t)h * n_q + (active ? qi : 0)) * D;
#pragma unroll
        for (int t = 0; t < D; ++t) {
            q[t] = qrow[t];
            o[t] = 0.0f;
        }
    }
    float m_run = -INFINITY, l_run = 0.0f;
    for (int e = 0; e < n_listed; ++e) {
        const int kb = sel_row[e];
        if (kb < 0) continue;  // uniform over the workgroup
        const int kend = min((kb + 1) * BK, L);
        for (int k0 = kb * BK; k0 < kend; k0 += TKF) {
            const int nk = min(TKF, kend - k0);
            __syncthreads();
            for (int x = tid; x < nk * (D / 4); x += blockDim.x) {
                const int row = x / (D / 4), c4 = x % (D / 4);
                *(f32x4 *)(Ks + row * D + 4 * c4) = *(const f32x4 *)(K + ((size_t)h * C + k0 + row) * D + 4 * c4);
                *(f32x4 *)(Vs + row * D + 4 * c4) = *(const f32x4 *)(V + ((size_t)h * C + k0 + row) * D + 4 * c4);
            }
            if (tid < nk) bias[tid] = cnt ? log2f((float)cnt[(size_t)h * C + k0 + tid]) : 0.0f;
            __syncthreads();
            float s[TKF];
            float mx = -INFINITY;
#pragma unroll
            for (int j = 0; j < TKF; ++j) {
                float acc = -INFINITY;
                if (j < nk) {
                    acc = 0.0f;
#pragma unroll
                    for (int t = 0; t < D; t += 4) {
                        const f32x4 kv = *(const f32x4 *)(Ks + j * D + t);
                        acc = fmaf(q[t], kv[0], acc);
                        acc = fmaf(q[t + 1], kv[1], acc);
                        acc = fmaf(q[t + 2], kv[2], acc);
                        acc = fmaf(q[t + 3], kv[3], acc);
                    }
                    acc = fmaf(acc, scale_log2, bias[j]);
                }
                s[j] = acc;
                mx = fmaxf(mx, acc);
            }
            const float m_new = fmaxf(m_run, mx);  // nk >= 1, so m_new is finite
            const float alpha = exp2f(m_run - m_new);
            l_run *= alpha;
#pragma unroll
            for (int t = 0; t < D; ++t) o[t] *= alpha;
#pragma unroll
            for (int j = 0; j < TKF; ++j) {
                if (j < nk) {
                    const float p = exp2f(s[j] - m_new);
                    l_run += p;
#pragma unroll
                    for (int t = 0; t < D; t += 4) {
                        const f32x4 vv = *(const f32x4 *)(Vs + j * D + t);
                        o[t] = fmaf(p, vv[0], o[t]);
                        o[t + 1] = fmaf(p, vv[1], o[t + 1]);
                        o[t + 2] = fmaf(p, vv[2], o[t + 2]);
                        o[t + 3] = fmaf(p, vv[3], o[t + 3]);
                    }
                }
            }
            m_run = m_new;
        }
    }
    if (active) {
        const float inv = l_run > 0.0f ? 1.0f / l_run : 0.0f;
        float *orow = O + ((size_t)h * n_q + qi) * D;
#pragma unroll
        for (int t = 0; t < D; ++t) orow[t] = o[t] * inv;
        if (lse) lse[(size_t)h * n_q + qi] = l_run > 0.0f ? (m_run + log2f(l_run)) * LN2 : -INFINITY;
    }
}

int launch_attn_bf16_d128(const void *Q, int n_q, const void *K, const void *V, const int32_t *cnt, const int32_t *len,
                          int H, int C, const int32_t *sel, const int32_t *nsel, int BQ, int bk_shift, int n_sel,
                          float scale_log2, void *O, float *lse, hipStream_t s);
int launch_attn_bf16_d128_pp(const void *Q, int n_q, const void *K, const void *V, const int32_t *cnt,
                             const int32_t *len, int H, int C, const int32_t *sel, const int32_t *nsel, int bk_shift,
                             int n_sel, float scale_log2, void *O, float *lse, hipStream_t s);

size_t attn_sk_ws_bytes();
int launch_attn_bf16_d128_sk(const void *Q, int n_q, const void *K, const void *V, const int32_t *cnt, const int32_t *len,
                             int H, int C, const int32_t *sel, const int32_t *nsel, int bk_shift, int n_sel,
                             float scale_log2, void *O, float *lse, void *ws, int full_per, hipStream_t s);

}  // namespace fastar

using namespace fastar;

static int sparse_attn_impl(const void *Q, int n_q, const void *K, const void *V, const int32_t *cnt,
                            const int32_t *len, int H, int C, int d, int dtype, const int32_t *sel,
                            const int32_t *nsel, int BQ, int BK, int n_sel, float scale, void *O, float *lse,
                            void *ws, size_t ws_bytes, void *stream);

extern "C" int sparse_attn_fwd(const void *Q, int n_q, const void *K, const void *V, const int32_t *cnt,
                               const int32_t *len, int H, int C, int d, int dtype, const int32_t *sel,
                               const int32_t *nsel, int BQ, int BK, int n_sel, float scale, void *O, float *lse,
                               void *stream) {
    return sparse_attn_impl(Q, n_q, K, V, cnt, len, H, C, d, dtype, sel, nsel, BQ, BK, n_sel, scale, O, lse, nullptr, 0,
                            stream);
}

extern "C" int sparse_attn_fwd_ws(const void *Q, int n_q, const void *K, const void *V, const int32_t *cnt,
                                  const int32_t *len, int H, int C, int d, int dtype, const int32_t *sel,
                                  const int32_t *nsel, int BQ, int BK, int n_sel, float scale, void *O, float *lse,
                                  void *ws, size_t ws_bytes, void *stream) {
    if (!ws || ((uintptr_t)ws & 255)) return FASTAR_ERR_INVALID_ARG;
    if (ws_bytes < attn_sk_ws_bytes()) return FASTAR_ERR_WORKSPACE;
    return sparse_attn_impl(Q, n_q, K, V, cnt, len, H, C, d, dtype, sel, nsel, BQ, BK, n_sel, scale, O, lse, ws, ws_bytes,
                            stream);
}

static int sparse_attn_impl(const void *Q, int n_q, const void *K, const void *V, const int32_t *cnt,
                               const int32_t *len, int H, int C, int d, int dtype, const int32_t *sel,
                               const int32_t *nsel, int BQ, int BK, int n_sel, float scale, void *O, float *lse,
                               void *ws, size_t ws_bytes, void *stream) {
    (void)ws_bytes;
    if (!Q || !K || !V || !len || !sel || !nsel || !O) return FASTAR_ERR_INVALID_ARG;
    if (H <= 0 || n_q <= 0 || C <= 0 || BQ <= 0 || BK <= 0 || n_sel <= 0) return FASTAR_ERR_INVALID_ARG;
    if (dtype != FASTAR_F32 && dtype != FASTAR_BF16) return FASTAR_ERR_INVALID_ARG;
    if (!(scale > 0.0f) || !(scale < INFINITY)) return FASTAR_ERR_INVALID_ARG;
    if (((uintptr_t)Q & 15) || ((uintptr_t)K & 15) || ((uintptr_t)V & 15) || ((uintptr_t)O & 15))
        return FASTAR_ERR_INVALID_ARG;
    if (d != 64 && d != 128) return FASTAR_ERR_UNSUPPORTED;
    const int n_qb = (n_q + BQ - 1) / BQ;
    hipStream_t s = (hipStream_t)stream;
    const float scale_log2 = scale * LOG2E;
    if (dtype == FASTAR_BF16) {
        if ((BQ != 64 && BQ != 128) || BK > 64 || (BK & (BK - 1)) != 0) return FASTAR_ERR_UNSUPPORTED;
        if ((unsigned long long)C * (unsigned long long)d * 2ull >= (1ull << 32)) return FASTAR_ERR_UNSUPPORTED;  // 32-bit row offsets
        int bk_shift = 0;
        while ((1 << bk_shift) < BK) ++bk_shift;
        const dim3 grid((unsigned)(((n_qb * H + 7) / 8) * 8));
#define FASTAR_ATTN(DD, NW)                                                                                       \
    hipLaunchKernelGGL((attn_bf16_kernel<DD, NW>), grid, dim3(NW * 64), 0, s, (const unsigned short *)Q,          \
                       (const unsigned short *)K, (const unsigned short *)V, cnt, len, sel, nsel, n_q, C, bk_shift, \
                       n_sel, n_qb, H, scale_log2, (unsigned short *)O, lse)
        // Two query blocks per workgroup in anti-phase (matrix | vector) on each SIMD; one workgroup fills a CU, so the
        // work comes in rounds of 512 query blocks: when the last round would be less than half full, the kernel with
        // one block per workgroup (two workgroups per CU, started as slots free up) finishes earlier.
        const int n_items = n_qb * H;
        // With a workspace, and more query blocks than the chip holds at once in a number that leaves a short last
        // round (an XCD holds 64 workgroups of the one-block kernel; a round that only a few of them take part in lasts
        // half as long as a full one, with most of the chip idle): the one-block kernel on whole rounds, then the query
        // blocks left over cut into equal shares of their tiles for all resident workgroups (long enough shares to pay for
        // the fragments and their combination).
        const int n_tiles = (int)(((long long)n_sel * BK + 63) / 64);
        const int full_per = attn_split_full_per(n_items, n_tiles);
        if (ws && d == 128 && BQ == 128 && full_per > 0)
            return launch_attn_bf16_d128_sk(Q, n_q, K, V, cnt, len, H, C, sel, nsel, bk_shift, n_sel, scale_log2, O, lse, ws,
                                            full_per, s);
        if (d == 128 && BQ == 128 && (n_items <= 512 || n_items % 512 == 0 || n_items % 512 >= 256))
            return launch_attn_bf16_d128_pp(Q, n_q, K, V, cnt, len, H, C, sel, nsel, bk_shift, n_sel, scale_log2, O, lse, s);
        if (d == 128)  // tuned path: direct-to-LDS tiles, LDS transpose loads
            return launch_attn_bf16_d128(Q, n_q, K, V, cnt, len, H, C, sel, nsel, BQ, bk_shift, n_sel, scale_log2, O, lse, s);
        if (BQ == 128) FASTAR_ATTN(64, 4);
        else FASTAR_ATTN(64, 2);
#undef FASTAR_ATTN
    } else {
        if (BQ > 128 || BK > 64) return FASTAR_ERR_UNSUPPORTED;
        const dim3 grid(n_qb, H);
        if (d == 128)
            hipLaunchKernelGGL(attn_f32_kernel<128>, grid, dim3(128), 0, s, (const float *)Q, (const float *)K,
                               (const float *)V, cnt, len, sel, nsel, n_q, C, BQ, BK, n_sel, n_qb, scale_log2,
                               (float *)O, lse);
        else
            hipLaunchKernelGGL(attn_f32_kernel<64>, grid, dim3(128), 0, s, (const float *)Q, (const float *)K,
                               (const float *)V, cnt, len, sel, nsel, n_q, C, BQ, BK, n_sel, n_qb, scale_log2,
                               (float *)O, lse);
    }
    FASTAR_LAUNCH_CHECK();
    return FASTAR_OK;
}
