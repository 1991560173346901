// Block-sparse attention, bf16, head dimension 128: two query blocks per workgroup in anti-phase.
//
// Same mathematics, operand layouts and data path as attention_d128.hip (transposed contractions,
// direct-to-LDS K/V tiles with XOR swizzle, LDS transpose loads for V^T, inline-assembly operand reads
// with explicit waits).  What differs is the schedule.  A SIMD of this chip runs matrix instructions of
// one wavefront and vector instructions of another at the same time, but two independent workgroups on
// a CU drift through their matrix (QK^T, PV) and vector (softmax) phases at random, and measured overlap
// is poor.  Here one workgroup holds TWO groups of wavefronts, each group owning one query block with its
// own selection list, K/V stages and row tables; wavefronts w and w + NWG share a SIMD.  Every tile is
// split into
//     X(t): O += P(t-1) V(t-1), then S(t) = K(t) Q^T        (matrix cores, ~32 instructions of 32 cycles)
//     Y(t): softmax of S(t) -> P(t), running max / sum      (vector ALUs, about as long)
// and the two groups are kept half a tile apart by a workgroup barrier per half step, so that on every
// SIMD one wavefront is in X while the other is in Y.  K tiles run one tile ahead of V tiles.
// Both phases are bound by what one wavefront can issue (a vector instruction every 5.4 cycles, measured), so
// Y carries as few instructions as possible; with key blocks of 64 rows (CONTIG) it has no row table at all.
#include <type_traits>

#include "common.hpp"

namespace fastar {

namespace d128pp {

#pragma clang diagnostic ignored "-Winline-asm"   // m0 is named as clobbered where the tile loads set it

constexpr int D = 128;
constexpr int TK = 64;                 // keys per tile
constexpr int ROWB = D * 2;            // bytes per K/V row
constexpr int TILEB = TK * ROWB;       // 16 KiB per tile
constexpr int GROUPB = 4 * TILEB;      // per group: K stage 0/1, V stage 0/1
constexpr float LN2 = 0.6931471805599453f;

typedef __attribute__((ext_vector_type(4))) short s16x4;
#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T *)(p))

struct __attribute__((aligned(16))) TileMeta {
    int idx[TK];     // cache row of each tile position (masked positions: row 0)
    float bias[TK];  // log2(cnt) of that row in units of raw scores (divided by scale * log2 e), -inf when masked
};

// dynamic LDS layout: [group 0: K0 K1 V0 V1][group 1: K0 K1 V0 V1][meta x4 of group 0][meta x4 of group 1]
constexpr int NMETA = 4;   // row tables in flight per group
constexpr int LDS_BYTES = 2 * GROUPB + 2 * NMETA * (int)sizeof(TileMeta);

template <int OFF>
__device__ __forceinline__ s16x4 lds_read_tr16(unsigned addr) {
    s16x4 r;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
    return r;
}
template <int OFF>
__device__ __forceinline__ bf16x8 lds_read_b128(unsigned addr) {
    bf16x8 r;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
    return r;
}
// K operands of 32 keys for the eight 16-coordinate steps; BASE = byte offset of the first row in the group's region.
template <int BASE>
__device__ __forceinline__ void read_k(bf16x8 (&f)[D / 16], const unsigned (&kaddr)[D / 16]) {
    f[0] = lds_read_b128<BASE>(kaddr[0]); f[1] = lds_read_b128<BASE>(kaddr[1]);
    f[2] = lds_read_b128<BASE>(kaddr[2]); f[3] = lds_read_b128<BASE>(kaddr[3]);
    f[4] = lds_read_b128<BASE>(kaddr[4]); f[5] = lds_read_b128<BASE>(kaddr[5]);
    f[6] = lds_read_b128<BASE>(kaddr[6]); f[7] = lds_read_b128<BASE>(kaddr[7]);
}
// Wait until at most eight LDS operations are outstanding: with one batch of eight reads issued after f, f has
// landed (LDS operations complete in order; anything else issued in between only makes the wait stricter).
__device__ __forceinline__ void wait_k_but8(bf16x8 (&f)[D / 16]) {
    asm volatile("s_waitcnt lgkmcnt(8)"
                 : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]), "+v"(f[4]), "+v"(f[5]), "+v"(f[6]), "+v"(f[7]));
}
__device__ __forceinline__ void wait_k(bf16x8 (&f)[D / 16]) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]), "+v"(f[4]), "+v"(f[5]), "+v"(f[6]), "+v"(f[7]));
}
// V^T operands of 32 keys (two steps of 16) for the four 32-column blocks.
template <int BASE>
__device__ __forceinline__ void read_vt(s16x4 (&f)[2][D / 32][2], const unsigned (&vaddr)[D / 32]) {
#define FASTAR_RD(ST, DB)                                                          \
    f[ST][DB][0] = lds_read_tr16<BASE + (16 * ST) * ROWB>(vaddr[DB]);               \
    f[ST][DB][1] = lds_read_tr16<BASE + (16 * ST + 8) * ROWB>(vaddr[DB]);
    FASTAR_RD(0, 0) FASTAR_RD(0, 1) FASTAR_RD(0, 2) FASTAR_RD(0, 3)
    FASTAR_RD(1, 0) FASTAR_RD(1, 1) FASTAR_RD(1, 2) FASTAR_RD(1, 3)
#undef FASTAR_RD
}
__device__ __forceinline__ void wait_vt(s16x4 (&f)[2][D / 32][2]) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(f[0][0][0]), "+v"(f[0][0][1]), "+v"(f[0][1][0]), "+v"(f[0][1][1]), "+v"(f[0][2][0]),
                   "+v"(f[0][2][1]), "+v"(f[0][3][0]), "+v"(f[0][3][1]), "+v"(f[1][0][0]), "+v"(f[1][0][1]),
                   "+v"(f[1][1][0]), "+v"(f[1][1][1]), "+v"(f[1][2][0]), "+v"(f[1][2][1]), "+v"(f[1][3][0]),
                   "+v"(f[1][3][1]));
}
// Wait until at most eight LDS operations are outstanding (one batch of eight issued after f).
__device__ __forceinline__ void wait_vt_but8(s16x4 (&f)[2][D / 32][2]) {
    asm volatile("s_waitcnt lgkmcnt(8)"
                 : "+v"(f[0][0][0]), "+v"(f[0][0][1]), "+v"(f[0][1][0]), "+v"(f[0][1][1]), "+v"(f[0][2][0]),
                   "+v"(f[0][2][1]), "+v"(f[0][3][0]), "+v"(f[0][3][1]), "+v"(f[1][0][0]), "+v"(f[1][0][1]),
                   "+v"(f[1][1][0]), "+v"(f[1][1][1]), "+v"(f[1][2][0]), "+v"(f[1][2][1]), "+v"(f[1][3][0]),
                   "+v"(f[1][3][1]));
}
__device__ __forceinline__ void pv_mfma(f32x16 (&o_acc)[D / 32], const s16x4 (&f)[2][D / 32][2],
                                        const bf16x8 (&pf)[2]) {
#pragma unroll
    for (int st = 0; st < 2; ++st)
#pragma unroll
        for (int db = 0; db < D / 32; ++db) {
            struct { s16x4 a, b; } pr = {f[st][db][0], f[st][db][1]};
            bf16x8 a;
            __builtin_memcpy(&a, &pr, 16);
            o_acc[db] = mfma_bf16_32x32x16(a, pf[st], o_acc[db]);
        }
}

// max(x[l], x[l ^ 32]) on the vector ALU (the lane-swap instruction of this chip), without a trip through the LDS
// queue, where it would wait behind the other group's operand reads.
__device__ __forceinline__ float max_across_halves(float x) {
    const unsigned u = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// Workgroup barrier that waits for this wavefront's LDS traffic but NOT for its outstanding global -> LDS tile
// loads (the fence of __syncthreads would drain those too and shorten the prefetch distance to half a tile).
// The scheduling fences keep register-only work of one phase from drifting across into the next.
__device__ __forceinline__ void wg_barrier() {
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

// NWG = wavefronts per group; a group owns a query block of 32*NWG queries.
// CONTIG = key blocks of 64 rows (bk_shift = 6): a tile is one selection entry, 64 consecutive cache rows.  Then there
// is no row table: every wavefront takes the entry from a register (one lane per entry of the list), a tile that lies
// wholly below len is loaded from one uniform base address with the row and chunk in the instructions' immediate
// offsets (any other tile row by row, rows at or beyond len redirected to row 0), and only the multiplicity bias
// goes through LDS.
// BIAS_X (with CONTIG): the bias row of a tile is written in the matrix phase, one step after its multiplicities were
// requested there, instead of at the head of the vector phase.  That shortens the vector phase (the longer one), but the
// compiler's wait for the multiplicities then also waits for the tile loads the vector phase in between has issued:
// good while those come from L2 / the memory-side cache, bad once the cache outgrows them.
template <int NWG, bool CONTIG, bool BIAS_X>
__global__ __launch_bounds__(2 * NWG * 64, 1) void attn_bf16_d128_pp_kernel(
    const unsigned short *__restrict__ Q, const unsigned short *__restrict__ K, const unsigned short *__restrict__ V,
    const int32_t *__restrict__ cnt, const int32_t *__restrict__ len, const int32_t *__restrict__ sel,
    const int32_t *__restrict__ nsel, int n_q, int C, int bk_shift, int n_sel, int n_qb, int H, float scale_log2,
    float inv_scale_log2, unsigned short *__restrict__ O, float *__restrict__ lse) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    constexpr int GT = NWG * 64;            // threads per group
    constexpr int IPW = (TK / 4) / NWG;     // 1-KiB direct-load instructions per wavefront and tensor

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = wave / NWG, gw = wave % NWG;   // group, wavefront within the group (both wave-uniform)
    const int gtid = tid - grp * GT;
    const int col = lane & 31, g = lane >> 5;

    // workgroup -> pair of consecutive (head, query block) items; XCD-contiguous ranges of pairs
    const int total = n_qb * H;
    const int pairs = (total + 1) / 2;
    int pair;
    {
        const int wg = blockIdx.x;
        const int per = (pairs + 7) / 8;
        pair = (wg & 7) * per + (wg >> 3);
        if (pair >= pairs) return;
    }
    auto tiles_of = [&](int item) -> int {   // uniform
        if (item >= total) return 0;
        const int hh = item / n_qb, bb = item % n_qb;
        const int Lh = min(len[hh], C);
        const int nl = Lh > 0 ? min(nsel[(size_t)hh * n_qb + bb], n_sel) : 0;
        return ((nl << bk_shift) + TK - 1) / TK;
    };
    const int nt0 = tiles_of(2 * pair), nt1 = tiles_of(2 * pair + 1);
    const int item = min(2 * pair + grp, total - 1);
    const bool valid = 2 * pair + grp < total;
    const int nt = grp == 0 ? nt0 : nt1;
    const int h = item / n_qb, b = item % n_qb;
    const int L = min(len[h], C);
    const int n_listed = (valid && L > 0) ? min(nsel[(size_t)h * n_qb + b], n_sel) : 0;
    const int32_t *sel_row = sel + ((size_t)h * n_qb + b) * n_sel;
    const int32_t *cnt_h = cnt ? cnt + (size_t)h * C : nullptr;
    const unsigned short *Kh = K + (size_t)h * C * D;
    const unsigned short *Vh = V + (size_t)h * C * D;

    unsigned char *gbase = lds + grp * GROUPB;
    unsigned char *kbuf = gbase;
    unsigned char *vbuf = gbase + 2 * TILEB;
    TileMeta *meta = (TileMeta *)(lds + 2 * GROUPB) + NMETA * grp;

    const int q_idx = b * (NWG * 32) + gw * 32 + col;
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
    // running softmax state per query (lanes l and l+32 hold the two key halves of query column l%32):
    // m_ref = reference maximum in raw score units, neg_ms = -m_ref * scale (0 while m_ref = -inf), l0/l1 = sums of P
    float m_ref = -INFINITY, neg_ms = 0.0f, l0 = 0.0f, l1 = 0.0f;
    const float tau_raw = 8.0f * inv_scale_log2;   // the reference may lag the true maximum by 8 octaves: P <= 256

    // direct global -> LDS loads of one tile of K or V: instruction i of this wavefront covers tile rows
    // 4*(gw*IPW+i) .. +3, lane l -> row +l/16, LDS chunk l%16, global chunk swizzled.  With IPW = 4 the row's
    // swizzle is the lane's own part XOR a constant of the instruction, so an address costs two vector operations
    // on a 32-bit byte offset from the head's (uniform) base.
    static_assert(IPW == 4, "swizzle constants below assume four instructions per wavefront");
    const int lrow = lane >> 4, lchunk = lane & 15;
    const unsigned kswz = (unsigned)(lchunk ^ lrow) << 4;          // K: chunk ^ (row & 15), row & 15 = 4 i + lrow
    const unsigned vswz = (unsigned)(lchunk ^ (lrow << 1)) << 4;   // V: chunk ^ 2 (row & 7), row & 7 = 4 (i & 1) + lrow
    auto tile_keys = [&](int (&keys)[IPW], const TileMeta &m) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < IPW; ++i) keys[i] = m.idx[4 * (gw * IPW + i) + lrow];
    };
    auto issue_keys = [&](const unsigned short *base, unsigned char *dst, const int (&keys)[IPW], auto is_v) __attribute__((always_inline)) {
        constexpr bool IS_V = decltype(is_v)::value;
#pragma unroll
        for (int i = 0; i < IPW; ++i) {
            const unsigned off = ((unsigned)keys[i] << 8) | (IS_V ? (vswz ^ (128u * (i & 1))) : (kswz ^ (64u * i)));
            const unsigned char *src = (const unsigned char *)base + off;
            __builtin_amdgcn_global_load_lds(src, LDS_PTR(unsigned, dst + (gw * IPW + i) * 1024), 16, 0, 0);
        }
    };
    auto issue_rows = [&](const unsigned short *base, unsigned char *dst, const TileMeta &m, auto is_v) __attribute__((always_inline)) {
        int keys[IPW];
        tile_keys(keys, m);
        issue_keys(base, dst, keys, is_v);
    };
    // ---- CONTIG: selection entries in a register, tiles by base address -------------------------------------------
    const unsigned lds_base = (unsigned)(size_t)LDS_PTR(unsigned char, lds);
    int sel_chunk = 0;
    int selv = -1;   // lane l: entry 64 * sel_chunk + l of the list
    if constexpr (CONTIG) {
        if (n_listed > 0) selv = sel_row[min(lane, n_listed - 1)];
        asm volatile("s_waitcnt vmcnt(0)" : "+v"(selv)::"memory");
    }
    // first row of tile t (uniform; -1: no such tile or a negative entry); tiles are asked for in rising order
    auto row0_of = [&](int t) __attribute__((always_inline)) -> int {
        if (t >= nt) return -1;
        if ((t >> 6) != sel_chunk) {
            sel_chunk = t >> 6;
            selv = sel_row[min(64 * sel_chunk + lane, n_listed - 1)];
            // waited for here, once per 64 tiles, so that the common path carries no wait for it
            asm volatile("s_waitcnt vmcnt(0)" : "+v"(selv)::"memory");
        }
        const int kb = __builtin_amdgcn_readlane(selv, t & 63);
        return kb >= 0 ? kb * TK : -1;
    };
    unsigned koff[IPW], voff[2];   // per-lane parts of a tile load: row within the instruction's four, swizzled chunk
#pragma unroll
    for (int i = 0; i < IPW; ++i) koff[i] = ((unsigned)lrow << 8) | (kswz ^ (64u * i));
#pragma unroll
    for (int i = 0; i < 2; ++i) voff[i] = ((unsigned)lrow << 8) | (vswz ^ (128u * i));
    // this wavefront's share (tile rows 16 gw .. 16 gw + 15) of the tile that starts at cache row row0
    auto issue_tile = [&](const unsigned short *base, unsigned char *dst, int row0, auto is_v) __attribute__((always_inline)) {
        constexpr bool IS_V = decltype(is_v)::value;
        if (row0 >= 0 && row0 + TK <= L) {
            // the immediate offset of a direct load moves the global and the LDS address alike: 1 KiB per instruction
            const unsigned char *tb =
                (const unsigned char *)base + ((size_t)(unsigned)(__builtin_amdgcn_readfirstlane(row0) + 4 * IPW * gw) << 8);
            const unsigned d = lds_base + (unsigned)(dst - lds) + gw * IPW * 1024;
            unsigned o0, o1, o2, o3;
            if constexpr (IS_V) { o0 = voff[0]; o1 = voff[1]; o2 = voff[0]; o3 = voff[1]; }
            else { o0 = koff[0]; o1 = koff[1]; o2 = koff[2]; o3 = koff[3]; }
            asm volatile("s_mov_b32 m0, %[d]\n\t"
                         "s_nop 0\n\t"
                         "global_load_lds_dwordx4 %[o0], %[b]\n\t"
                         "global_load_lds_dwordx4 %[o1], %[b] offset:1024\n\t"
                         "global_load_lds_dwordx4 %[o2], %[b] offset:2048\n\t"
                         "global_load_lds_dwordx4 %[o3], %[b] offset:3072"
                         :
                         : [d] "s"(d), [b] "s"(tb), [o0] "v"(o0), [o1] "v"(o1), [o2] "v"(o2), [o3] "v"(o3)
                         : "memory", "m0");
        } else {
            int keys[IPW];
#pragma unroll
            for (int i = 0; i < IPW; ++i) {
                const int row = row0 + 4 * (gw * IPW + i) + lrow;
                keys[i] = (row0 >= 0 && row < L) ? row : 0;   // masked rows fetch row 0, which is live
            }
            issue_keys(base, dst, keys, is_v);
        }
    };
    // bias row of tile t: log2 of the multiplicity c of tile position gtid (threads gtid < 64 of the group)
    auto write_bias = [&](int t, int row0, int c) __attribute__((always_inline)) {
        const int row = row0 + gtid;
        const bool live = row0 >= 0 && row < L;
        meta[t & (NMETA - 1)].bias[gtid] = live ? (cnt_h ? __log2f((float)c) * inv_scale_log2 : 0.0f) : -INFINITY;
    };
    auto cnt_of = [&](int row0) __attribute__((always_inline)) -> int {
        const int row = row0 + gtid;
        return (cnt_h && row0 >= 0 && row < L) ? cnt_h[row] : 1;
    };
    int r1 = -1, r2 = -1, r3 = -1, r4 = -1;   // first rows of tiles t+1 .. t+4 as seen from X(t) and Y(t)

    // row tables: position p of tile `tile` (threads gtid < 64 of the group)
    auto sel_entry = [&](int tile) __attribute__((always_inline)) -> int {
        const int entry = (tile * TK + gtid) >> bk_shift;
        return (gtid < TK && entry < n_listed) ? sel_row[entry] : -1;
    };
    auto key_of = [&](int kb, int tile) __attribute__((always_inline)) -> int {
        int key = -1;
        if (kb >= 0) {
            key = (kb << bk_shift) + ((tile * TK + gtid) & ((1 << bk_shift) - 1));
            if (key >= L) key = -1;
        }
        return key;
    };
    auto write_meta = [&](int tile, int key, int c) __attribute__((always_inline)) {
        if (gtid < TK) {
            TileMeta &m = meta[tile & (NMETA - 1)];
            m.idx[gtid] = key >= 0 ? key : 0;
            m.bias[gtid] = key >= 0 ? (cnt_h ? __log2f((float)c) * inv_scale_log2 : 0.0f) : -INFINITY;
        }
    };
    // Row tables run ahead of the tile loads: Y(t) writes the table of tile t+3 from values it requested during
    // Y(t-1) (their loads are covered by the wait at the head of every Y), and requests those of tile t+4.
    int key_n = -1, cnt_n = 1;   // row and multiplicity of this thread's position in the next table to write
    int kb_ahead = -1;           // selection entry of this thread's position in the table after that
    if constexpr (CONTIG) {
        const int r0 = row0_of(0);
        r1 = row0_of(1);
        r2 = row0_of(2);
        r3 = row0_of(3);
        if (nt > 0 && gw == 0) {
            write_bias(0, r0, cnt_of(r0));
            write_bias(1, r1, cnt_of(r1));
            write_bias(2, r2, cnt_of(r2));
            if constexpr (BIAS_X) cnt_n = cnt_of(r3);
            else write_bias(3, r3, cnt_of(r3));
        }
        __syncthreads();
        if (nt > 0) {   // K(0), K(1) -> K stages 0, 1; V(0) -> V stage 0
            issue_tile(Kh, kbuf, r0, std::false_type{});
            if (nt > 1) issue_tile(Kh, kbuf + TILEB, r1, std::false_type{});
            issue_tile(Vh, vbuf, r0, std::true_type{});
        }
    } else {
        if (nt > 0) {
#pragma unroll
            for (int tt = 0; tt < 3; ++tt) {
                const int key = key_of(tt < nt ? sel_entry(tt) : -1, tt);
                write_meta(tt, key, (key >= 0 && cnt_h) ? cnt_h[key] : 1);
            }
            if (nt > 3) {
                key_n = key_of(sel_entry(3), 3);
                if (key_n >= 0 && cnt_h) cnt_n = cnt_h[key_n];
                if (nt > 4) kb_ahead = sel_entry(4);
            }
        }
        __syncthreads();
        if (nt > 0) {   // K(0), K(1) -> K stages 0, 1; V(0) -> V stage 0
            issue_rows(Kh, kbuf, meta[0], std::false_type{});
            if (nt > 1) issue_rows(Kh, kbuf + TILEB, meta[1], std::false_type{});
            issue_rows(Vh, vbuf, meta[0], std::true_type{});
        }
    }

    // per-lane LDS addresses (see attention_d128.hip), including the group's base
    const unsigned kbuf_lds = (unsigned)(size_t)LDS_PTR(unsigned char, kbuf);
    unsigned kaddr[D / 16];
#pragma unroll
    for (int s = 0; s < D / 16; ++s) kaddr[s] = kbuf_lds + col * ROWB + (((2 * s + g) ^ (col & 15)) << 4);
    const int s16 = lane & 15, l16 = lane >> 4;
    const int vrow_in = 4 * (l16 >> 1) + (s16 >> 2);
    const unsigned vbuf_lds = (unsigned)(size_t)LDS_PTR(unsigned char, vbuf);
    unsigned vaddr[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
        vaddr[db] = vbuf_lds + vrow_in * ROWB +
                    (((4 * db + 2 * (l16 & 1) + ((s16 & 3) >> 1)) ^ ((vrow_in & 7) << 1)) << 4) + (s16 & 1) * 8;

    f32x16 s_acc[2];
    bf16x8 pf[2][2];
    // The score accumulators start from the keys' bias (a per-lane pattern: register v is key row 8(v/4)+4g+v%4),
    // so K Q^T lands on top of it and masking / multiplicity cost no vector instruction.
    auto load_bias = [&](int t) __attribute__((always_inline)) {
        const float *bias = meta[t & (NMETA - 1)].bias;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const f32x4 bv = *(const f32x4 *)(&bias[32 * kb + 8 * q4 + 4 * g]);
#pragma unroll
                for (int e = 0; e < 4; ++e) s_acc[kb][4 * q4 + e] = bv[e];
            }
    };

    // X(t), t = 0 .. nt: O += P(t-1) V(t-1) (PV: t > 0), S(t) = bias + K(t) Q^T (QK: t < nt), tile maximum of S(t).
    // The first half of V(t-1) is already in registers (va, read at the end of Y(t-1)), so the matrix cores start
    // at once and cover the remaining operand reads.  K(t) sits in K stage t & 1 and V(t) in V stage t & 1;
    // kaddr / vaddr point at the stage to read and are moved to the other stage after use.
    s16x4 va[2][D / 32][2];
    float mx_tile = -INFINITY;   // per query: maximum of S(t) over the tile, handed from X(t) to Y(t)
    auto phase_x = [&](int t, auto pv_c, auto qk_c) __attribute__((always_inline)) {
        constexpr bool PV = decltype(pv_c)::value, QK = decltype(qk_c)::value;
        __builtin_amdgcn_s_setprio(2);   // the wavefront feeding the matrix cores goes first on its SIMD
        s16x4 vb[2][D / 32][2];
        bf16x8 ka[D / 16], kb2[D / 16];
        if constexpr (PV) read_vt<32 * ROWB>(vb, vaddr);     // V(t-1), keys 32..63 (keys 0..31 are in va)
        if constexpr (QK) read_k<0>(ka, kaddr);              // K(t), keys 0..31
        if constexpr (PV) pv_mfma(o_acc, va, pf[0]);
        if constexpr (CONTIG && QK) {
            // here rather than in Y, which is the longer phase: first row of tile t+4 and the request for its
            // multiplicities (BIAS_X: after the bias row of tile t+3, whose multiplicities X(t-1) requested; otherwise
            // the row of tile t+4 is written at the head of Y(t), behind the wait for every outstanding load that opens it)
            if constexpr (BIAS_X) {
                if (gw == 0 && t + 3 < nt) write_bias(t + 3, r3, cnt_n);
            }
            r4 = row0_of(t + 4);
            if (gw == 0) cnt_n = cnt_of(r4);
        }
        if constexpr (PV) {
            if constexpr (QK) wait_vt_but8(vb); else wait_vt(vb);
            pv_mfma(o_acc, vb, pf[1]);
#pragma unroll
            for (int db = 0; db < D / 32; ++db) vaddr[db] += (t & 1) ? TILEB : -TILEB;   // V(t-1) -> V(t)
        }
        if constexpr (QK) {
            load_bias(t);
            read_k<32 * ROWB>(kb2, kaddr);                   // keys 32..63
            wait_k_but8(ka);
#pragma unroll
            for (int s = 0; s < D / 16; ++s) s_acc[0] = mfma_bf16_32x32x16(ka[s], qf[s], s_acc[0]);
            wait_k(kb2);
            // the scores of keys 0..31 are complete: their maximum is taken under the products of keys 32..63
            __builtin_amdgcn_sched_barrier(0);
            float mx = s_acc[0][0];
#pragma unroll
            for (int s = 0; s < D / 16; ++s) {
                s_acc[1] = mfma_bf16_32x32x16(kb2[s], qf[s], s_acc[1]);
                if (s > 0) mx = fmaxf(mx, s_acc[0][2 * s]);
                mx = fmaxf(mx, s_acc[0][2 * s + 1]);
                kaddr[s] += (t & 1) ? -TILEB : TILEB;   // K(t) -> K(t+1)
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s_acc[1][v]);
            mx_tile = max_across_halves(mx);
            // all of it exists before the barrier: pure arithmetic would otherwise be free to sink past it
            asm volatile("" : "+v"(s_acc[0]), "+v"(s_acc[1]), "+v"(mx_tile));
        }
        __builtin_amdgcn_s_setprio(0);
    };
    // Y(t), t = 0 .. nt-1: everything that is not a matrix instruction.  Row table of tile t+3; loads of K(t+2) and
    // V(t+1) into the stages X(t) has just consumed; P(t) = exp2(scale * (S(t) - m_ref)) as bf16 operands and the
    // running sums; then, for X(t+1), the first half of V(t) into va (last, so that these reads do not queue up in
    // front of the other group's operand reads).
    // m_ref follows the running maximum lazily: O and the sums are rescaled only when some query of the wavefront
    // exceeds its reference by more than tau, which after the first tiles is rare; the result is the same softmax
    // (any reference cancels in O / l), P just ranges up to 2^8 instead of 1.
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    auto phase_y = [&](int t) __attribute__((always_inline)) {
        int kk[IPW], vk[IPW];
        if constexpr (CONTIG) {
            if constexpr (!BIAS_X) {
                if (gw == 0 && t + 4 < nt) write_bias(t + 4, r4, cnt_n);   // requested during X(t)
            }
        } else {
            if (t + 3 < nt) write_meta(t + 3, key_n, cnt_n);
            key_n = -1;
            cnt_n = 1;
            int kb_next = -1;
            if (t + 4 < nt) {
                key_n = key_of(kb_ahead, t + 4);
                if (key_n >= 0 && cnt_h) cnt_n = cnt_h[key_n];
                if (t + 5 < nt) kb_next = sel_entry(t + 5);
            }
            kb_ahead = kb_next;
            // row lists of the two tiles to fetch: read now, used after the exponentials (their LDS round trip queues
            // behind the other group's operand reads)
            tile_keys(kk, meta[(t + 2 < nt ? t + 2 : t) & (NMETA - 1)]);
            tile_keys(vk, meta[(t + 1 < nt ? t + 1 : t) & (NMETA - 1)]);
        }
        const float mx = mx_tile;
        if (__any(mx > m_ref + tau_raw)) {   // wave-uniform
            const float m_new = fmaxf(m_ref, mx);
            const float alpha = m_ref == -INFINITY ? 0.0f : __builtin_amdgcn_exp2f((m_ref - m_new) * scale_log2);
            m_ref = m_new;
            neg_ms = m_new == -INFINITY ? 0.0f : -m_new * scale_log2;
            l0 *= alpha;
            l1 *= alpha;
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) o_acc[db][v] *= alpha;
        }
        bf16x2 ones;
        ones[0] = (__bf16)1.0f;
        ones[1] = (__bf16)1.0f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                if (kb == 1 && hh == 0) {   // half way (the row lists have arrived by now)
                    if constexpr (CONTIG) {
                        if (t + 2 < nt) issue_tile(Kh, kbuf + (t & 1) * TILEB, r2, std::false_type{});
                        if (t + 1 < nt) issue_tile(Vh, vbuf + ((t + 1) & 1) * TILEB, r1, std::true_type{});
                    } else {
                        if (t + 2 < nt) issue_keys(Kh, kbuf + (t & 1) * TILEB, kk, std::false_type{});
                        if (t + 1 < nt) issue_keys(Vh, vbuf + ((t + 1) & 1) * TILEB, vk, std::true_type{});
                    }
                }
                bf16x2 pr[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float p0 = __builtin_amdgcn_exp2f(fmaf(s_acc[kb][8 * hh + 2 * j], scale_log2, neg_ms));
                    const float p1 = __builtin_amdgcn_exp2f(fmaf(s_acc[kb][8 * hh + 2 * j + 1], scale_log2, neg_ms));
                    pr[j][0] = (__bf16)p0;
                    pr[j][1] = (__bf16)p1;
                    // the sums take the rounded P, the values the PV product sees
                    if (j & 1) l1 = __builtin_amdgcn_fdot2_f32_bf16(pr[j], ones, l1, false);
                    else l0 = __builtin_amdgcn_fdot2_f32_bf16(pr[j], ones, l0, false);
                }
                __builtin_memcpy(&pf[kb][hh], pr, 16);
            }
        // P exists before the operand reads below are issued (and so before the barrier)
        asm volatile("" : "+v"(pf[0][0]), "+v"(pf[0][1]), "+v"(pf[1][0]), "+v"(pf[1][1]), "+v"(l0), "+v"(l1));
        read_vt<0>(va, vaddr);           // V(t), keys 0..31, for X(t+1)
        wait_vt(va);
        if constexpr (CONTIG) {
            r1 = r2;
            r2 = r3;
            r3 = r4;
        }
    };

    // Half steps.  A group with nt tiles runs X(0) Y(0) X(1) Y(1) ... Y(nt-1) X(nt), one workgroup barrier
    // before each.  Group 1 takes one idle barrier first, which puts the groups in anti-phase; afterwards each
    // group pads with idle barriers so that every wavefront passes the same number of them.  The barrier before
    // a Y also publishes the tiles whose loads the previous Y started (K(t+1), V(t)): each wavefront first waits
    // for its own shares of them.
    const int n_bar = max(nt0 > 0 ? 2 * nt0 + 1 : 0, nt1 > 0 ? 2 * nt1 + 2 : 1);
    int done = 0;
    if (grp == 1) { wg_barrier(); done = 1; }
    auto enter_landed = [&]() __attribute__((always_inline)) {
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
        wg_barrier();
    };
    if (nt > 0) {
        enter_landed();
        phase_x(0, std::false_type{}, std::true_type{});
        for (int t = 0; t < nt - 1; ++t) {
            enter_landed();
            phase_y(t);
            wg_barrier();
            phase_x(t + 1, std::true_type{}, std::true_type{});
        }
        enter_landed();
        phase_y(nt - 1);
        wg_barrier();
        phase_x(nt, std::true_type{}, std::false_type{});
        done += 2 * nt + 1;
    }
    for (; done < n_bar; ++done) wg_barrier();

    // epilogue: normalise, transpose through the group's own LDS region, store rows coalesced
    const float l_lane = l0 + l1;
    const float l_tot = l_lane + shfl_xor(l_lane, 32);
    const float inv = l_tot > 0.0f ? 1.0f / l_tot : 0.0f;
    __syncthreads();
    constexpr int OSTR = D + 8;  // bf16 elements per staged row (16-byte pad)
    unsigned short *Os = (unsigned short *)gbase + (size_t)gw * 32 * OSTR;
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
    if (valid) {
        const int rr = lane >> 4, cc = lane & 15;
#pragma unroll
        for (int it = 0; it < 8; ++it) {
            const int r = it * 4 + rr;
            const int qi = b * (NWG * 32) + gw * 32 + r;
            if (qi < n_q) *(u32x4 *)(O + ((size_t)h * n_q + qi) * D + cc * 8) = *(const u32x4 *)(Os + r * OSTR + cc * 8);
        }
        if (lse && g == 0 && q_idx < n_q)
            lse[(size_t)h * n_q + q_idx] = l_tot > 0.0f ? (m_ref * scale_log2 + __log2f(l_tot)) * LN2 : -INFINITY;
    }
}

}  // namespace d128pp

// more than 64 KiB of LDS per workgroup has to be requested once per kernel and device
int attn_d128_pp_setup() {
    using namespace d128pp;
    static DeviceOnce once;
    return once.run([](int) {
        for (const void *f : {(const void *)attn_bf16_d128_pp_kernel<4, false, false>,
                              (const void *)attn_bf16_d128_pp_kernel<4, true, false>,
                              (const void *)attn_bf16_d128_pp_kernel<4, true, true>})
            if (hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES) != hipSuccess)
                return FASTAR_ERR_HIP;
        return FASTAR_OK;
    });
}

// Launcher used by sparse_attn_fwd for bf16, d = 128, BQ = 128.
int launch_attn_bf16_d128_pp(const void *Q, int n_q, const void *K, const void *V, const int32_t *cnt,
                             const int32_t *len, int H, int C, const int32_t *sel, const int32_t *nsel, int bk_shift,
                             int n_sel, float scale_log2, void *O, float *lse, hipStream_t s) {
    using namespace d128pp;
    if (const int rc = attn_d128_pp_setup(); rc != FASTAR_OK) return rc;
    const int n_qb = (n_q + 127) / 128;
    const int pairs = (n_qb * H + 1) / 2;
    const dim3 grid((unsigned)(((pairs + 7) / 8) * 8));
#define FASTAR_PP(CONTIG, BIAS_X)                                                                                  \
    hipLaunchKernelGGL((attn_bf16_d128_pp_kernel<4, CONTIG, BIAS_X>), grid, dim3(512), LDS_BYTES, s,                \
                       (const unsigned short *)Q, (const unsigned short *)K, (const unsigned short *)V, cnt, len, sel, \
                       nsel, n_q, C, bk_shift, n_sel, n_qb, H, scale_log2, 1.0f / scale_log2, (unsigned short *)O, lse)
    // key blocks of 64 rows: tiles by base address; K and V of all heads within reach of the 256 MB memory-side cache:
    // the bias rows are written in the matrix phase
    const bool cache_resident = (size_t)H * (size_t)C * D * 2 * 2 <= ((size_t)256 << 20);
    if (bk_shift == 6 && cache_resident) FASTAR_PP(true, true);
    else if (bk_shift == 6) FASTAR_PP(true, false);
    else FASTAR_PP(false, false);
#undef FASTAR_PP
    if (hipGetLastError() != hipSuccess) return FASTAR_ERR_HIP;
    return FASTAR_OK;
}

}  // namespace fastar
