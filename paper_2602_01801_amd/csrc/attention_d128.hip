// Block-sparse attention, bf16, head dimension 128: the tuned path of sparse_attn_fwd.
//
// Same mathematics and the same "transposed" formulation as the generic kernel in attention.hip
// (S^T = K Q^T, O^T = V^T P^T, every per-query quantity in one lane), with a leaner data path:
//   * K and V tiles (64 gathered rows x 256 bytes) go from global memory straight into LDS with
//     16-byte direct loads: no staging registers, no VALU work, two LDS stages so that the loads
//     of tile t+1 fly while tile t is consumed, one workgroup barrier per tile;
//   * rows are stored unpadded and XOR-swizzled at 16-byte granularity (the swizzle is applied to
//     the global address each lane fetches, so it costs nothing): K chunk c of row r sits at chunk
//     c ^ (r & 15), V chunk c of row r at chunk c ^ (2 (r & 7)); both read patterns below are
//     bank-conflict free;
//   * the V^T operand is read from the row-major V tile with the LDS transpose load
//     (ds_read_b64_tr_b16): in each group of 16 lanes, lane 4q+m receives element m of the 8-byte
//     pieces addressed by lanes q, q+4, q+8, q+12, i.e. four consecutive keys of one value column;
//   * masked rows (padding of the selection list, slots beyond len) fetch row 0 of the head, which
//     is live, and carry a -inf bias, so they contribute exactly zero;
//   * the running-maximum rescale of O is skipped when no lane of the wavefront saw a new maximum.
#include <limits.h>

#include <type_traits>

#include "common.hpp"

namespace fastar {

namespace d128 {

constexpr int D = 128;
constexpr int TK = 64;                 // keys per tile
constexpr int ROWB = D * 2;            // bytes per K/V row
constexpr int TILEB = TK * ROWB;       // 16 KiB per tile
constexpr float LN2 = 0.6931471805599453f;

typedef __attribute__((ext_vector_type(4))) short s16x4;
#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T *)(p))

struct __attribute__((aligned(16))) TileMeta {
    int idx[TK];     // cache row of each tile position (masked positions: row 0)
    float bias[TK];  // log2(cnt) of that row in units of raw scores (divided by scale * log2 e), -inf when masked
};

__device__ __forceinline__ void fill_meta(TileMeta &m, int t, const int32_t *__restrict__ sel_row, int n_listed,
                                          int bk_shift, int L, const int32_t *__restrict__ cnt_h,
                                          float inv_scale_log2) {
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
        if (key >= 0) bias = cnt_h ? __log2f((float)cnt_h[key]) * inv_scale_log2 : 0.0f;
        m.idx[p] = key >= 0 ? key : 0;
        m.bias[p] = bias;
    }
}


// LDS transpose load issued as inline assembly: the compiler then neither serialises it against the
// direct-to-LDS tile loads in flight nor waits for it; wait_vt() below does, explicitly.
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

// K operands of 32 keys for the eight 16-coordinate steps.  BASE = byte offset of the first row inside the K region.
template <int BASE>
__device__ __forceinline__ void read_k(bf16x8 (&f)[D / 16], const unsigned (&kaddr)[D / 16]) {
    f[0] = lds_read_b128<BASE>(kaddr[0]); f[1] = lds_read_b128<BASE>(kaddr[1]);
    f[2] = lds_read_b128<BASE>(kaddr[2]); f[3] = lds_read_b128<BASE>(kaddr[3]);
    f[4] = lds_read_b128<BASE>(kaddr[4]); f[5] = lds_read_b128<BASE>(kaddr[5]);
    f[6] = lds_read_b128<BASE>(kaddr[6]); f[7] = lds_read_b128<BASE>(kaddr[7]);
}
__device__ __forceinline__ void wait_k(bf16x8 (&f)[D / 16]) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]), "+v"(f[4]), "+v"(f[5]), "+v"(f[6]), "+v"(f[7]));
}

// V^T operands of 32 keys (two steps of 16) for the four 32-column blocks: f[step][db][0|1] are the two
// 4-key halves of one A operand.  BASE = byte offset of the first of the 32 rows inside the V region.
template <int BASE>
__device__ __forceinline__ void read_vt(s16x4 (&f)[2][D / 32][2], const unsigned (&vaddr)[D / 32]) {
#define FASTAR_RD(ST, DB)                                                          \
    f[ST][DB][0] = lds_read_tr16<BASE + (16 * ST) * ROWB>(vaddr[DB]);               \
    f[ST][DB][1] = lds_read_tr16<BASE + (16 * ST + 8) * ROWB>(vaddr[DB]);
    FASTAR_RD(0, 0) FASTAR_RD(0, 1) FASTAR_RD(0, 2) FASTAR_RD(0, 3)
    FASTAR_RD(1, 0) FASTAR_RD(1, 1) FASTAR_RD(1, 2) FASTAR_RD(1, 3)
#undef FASTAR_RD
}

// Wait until every LDS read issued so far has returned; the operands tie the wait to the fragments.
__device__ __forceinline__ void wait_vt(s16x4 (&f)[2][D / 32][2]) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(f[0][0][0]), "+v"(f[0][0][1]), "+v"(f[0][1][0]), "+v"(f[0][1][1]), "+v"(f[0][2][0]),
                   "+v"(f[0][2][1]), "+v"(f[0][3][0]), "+v"(f[0][3][1]), "+v"(f[1][0][0]), "+v"(f[1][0][1]),
                   "+v"(f[1][1][0]), "+v"(f[1][1][1]), "+v"(f[1][2][0]), "+v"(f[1][2][1]), "+v"(f[1][3][0]),
                   "+v"(f[1][3][1]));
}

// O^T += V^T P^T for 32 keys: two steps of 16 keys, four 32-column blocks each.
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

// dynamic LDS layout: [K stage 0][K stage 1][V stage 0][V stage 1][meta x3]
constexpr int LDS_BYTES = 4 * TILEB + 3 * (int)sizeof(TileMeta);

constexpr int PART_O_FLOATS = (D / 32) * 16 * 64;              // O^T accumulators of one wavefront
constexpr int PART_FLOATS = 4 * (PART_O_FLOATS + 2 * 64);      // one fragment of a query block (4 wavefronts)
constexpr int SK_WORKGROUPS = 512;                             // two resident workgroups per CU
static_assert(PART_O_FLOATS == ATTN_PART_O_FLOATS && PART_FLOATS == ATTN_PART_FLOATS && SK_WORKGROUPS == ATTN_SHARE_WORKGROUPS,
              "fragment layout shared with the 8-bit kernel");

// One query block (h, b) over the tiles [t_begin, t_end) of its selection list (t_end may lie beyond the list: it is
// clipped).  part == nullptr: the block's output rows and lse are written.  Otherwise the fragment's unnormalised
// result goes to `part`: O^T accumulators as they sit in registers ([wave][db][v][lane] floats), then the reference
// maxima and the row sums ([wave][lane] each), for attn_combine_kernel.  All NW * 64 threads of a workgroup.
template <int NW>
__device__ __forceinline__ void attend_item(
    const unsigned short *__restrict__ Q, const unsigned short *__restrict__ K, const unsigned short *__restrict__ V,
    const int32_t *__restrict__ cnt, const int32_t *__restrict__ len, const int32_t *__restrict__ sel,
    const int32_t *__restrict__ nsel, int n_q, int C, int bk_shift, int n_sel, int n_qb, float scale_log2,
    float inv_scale_log2, unsigned short *__restrict__ O, float *__restrict__ lse, unsigned char *lds, int h, int b,
    int t_begin, int t_end, float *__restrict__ part) {
    unsigned char *kbuf = lds;
    unsigned char *vbuf = lds + 2 * TILEB;
    TileMeta *meta = (TileMeta *)(lds + 4 * TILEB);
    constexpr int IPW = (TK / 4) / NW;  // 1-KiB direct-load instructions per wavefront and tensor
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, kept in a scalar register
    const int col = lane & 31, g = lane >> 5;
    const int L = min(len[h], C);
    const int n_listed = L > 0 ? min(nsel[(size_t)h * n_qb + b], n_sel) : 0;
    const int32_t *sel_row = sel + ((size_t)h * n_qb + b) * n_sel;
    const int32_t *cnt_h = cnt ? cnt + (size_t)h * C : nullptr;
    const unsigned short *Kh = K + (size_t)h * C * D;
    const unsigned short *Vh = V + (size_t)h * C * D;
    const int nt = min(((n_listed << bk_shift) + TK - 1) / TK, t_end);   // end of this fragment
    const int t0 = min(t_begin, nt);

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
    // running softmax state per query (lanes l and l+32 hold the two key halves of query column l%32):
    // m_ref = reference maximum in raw score units, neg_ms = -m_ref * scale (0 while m_ref = -inf), l0/l1 = sums of P
    float m_ref = -INFINITY, neg_ms = 0.0f, l0 = 0.0f, l1 = 0.0f;
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

    // direct global -> LDS loads of one tile: instruction i of this wavefront covers tile rows
    // 4*(wave*IPW+i) .. +3, lane l -> row +l/16, LDS chunk l%16, global chunk swizzled
    const int lrow = lane >> 4, lchunk = lane & 15;
    auto issue_loads = [&](const TileMeta &m, int stage) {
        int keys[IPW];
#pragma unroll
        for (int i = 0; i < IPW; ++i) keys[i] = m.idx[4 * (wave * IPW + i) + lrow];
#pragma unroll
        for (int i = 0; i < IPW; ++i) {
            const int inst = wave * IPW + i;
            const int row = 4 * inst + lrow;
            const unsigned short *ksrc = Kh + (size_t)keys[i] * D + ((lchunk ^ (row & 15)) << 3);
            const unsigned short *vsrc = Vh + (size_t)keys[i] * D + ((lchunk ^ ((row & 7) << 1)) << 3);
            __builtin_amdgcn_global_load_lds(ksrc, LDS_PTR(unsigned, kbuf + stage * TILEB + inst * 1024), 16, 0, 0);
            __builtin_amdgcn_global_load_lds(vsrc, LDS_PTR(unsigned, vbuf + stage * TILEB + inst * 1024), 16, 0, 0);
        }
    };

    // Row tables are built two tiles ahead by the first 64 threads.  Their two dependent global loads
    // (selection entry, then multiplicity of the row it names) are split over two iterations and
    // issued BEFORE the tile loads of the iteration, and consumed at its end: memory operations
    // retire in order, so waiting for them any earlier would also wait for the tile in flight.
    auto sel_entry = [&](int tile) -> int {
        const int entry = (tile * TK + tid) >> bk_shift;
        return (tid < TK && entry < n_listed) ? sel_row[entry] : -1;
    };
    auto key_of = [&](int kb, int tile) -> int {
        int key = -1;
        if (kb >= 0) {
            key = (kb << bk_shift) + ((tile * TK + tid) & ((1 << bk_shift) - 1));
            if (key >= L) key = -1;
        }
        return key;
    };
    int kb_ahead = -1;  // selection entry of this thread's position in tile t+2
    if (nt > t0) {
        fill_meta(meta[t0 % 3], t0, sel_row, n_listed, bk_shift, L, cnt_h, inv_scale_log2);
        if (nt > t0 + 1) fill_meta(meta[(t0 + 1) % 3], t0 + 1, sel_row, n_listed, bk_shift, L, cnt_h, inv_scale_log2);
        if (nt > t0 + 2) kb_ahead = sel_entry(t0 + 2);
        __syncthreads();
        issue_loads(meta[t0 % 3], 0);
    }
    // Per-lane LDS byte offsets that do not depend on the tile.  XOR with a per-lane constant permutes
    // aligned groups of chunks, so every fragment address is (per-lane register) + (compile-time offset).
    //   K fragment (kb, s): row 32kb+col, logical chunk 2s+g -> chunk (2s+g) ^ (col & 15)
    //   V^T fragment (kstep, db): 16-lane group grp = lane/16 -> g = grp/2, column half = grp%2, s16 = lane%16;
    //     row kbase + 4g + s16/4 (+8), logical chunk 4db + 2*(grp%2) + (s16%4)/2, byte (s16%2)*8,
    //     swizzle 2*(row & 7) = 2*((4g + s16/4) & 7) for both rows
    const unsigned kbuf_lds = (unsigned)(size_t)LDS_PTR(unsigned char, kbuf);
    unsigned kaddr[D / 16];
#pragma unroll
    for (int s = 0; s < D / 16; ++s) kaddr[s] = kbuf_lds + col * ROWB + (((2 * s + g) ^ (col & 15)) << 4);
    const int s16 = lane & 15, grp = lane >> 4;
    const int vrow_in = 4 * (grp >> 1) + (s16 >> 2);
    const unsigned vbuf_lds = (unsigned)(size_t)LDS_PTR(unsigned char, vbuf);
    unsigned vaddr[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
        vaddr[db] = vbuf_lds + vrow_in * ROWB +
                    (((4 * db + 2 * (grp & 1) + ((s16 & 3) >> 1)) ^ ((vrow_in & 7) << 1)) << 4) + (s16 & 1) * 8;

    // A wavefront whose 32 queries all lie beyond n_q (the ragged last block of a head) still loads its share of every
    // tile and meets the barriers, but reads no operands and computes nothing.
    auto tile_step = [&](int t, auto stage_c, auto active_c) {
        constexpr int STAGE = decltype(stage_c)::value;
        constexpr bool ACTIVE = decltype(active_c)::value;
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wavefront's share of tile t has landed
        __syncthreads();                     // ... and everyone else's; tile t-1 fully consumed
        // row table of tile t+2, first half: issue its loads now
        int key2 = -1, cnt2 = 1, kb3 = -1;
        if (t + 2 < nt) {
            key2 = key_of(kb_ahead, t + 2);
            if (key2 >= 0 && cnt_h) cnt2 = cnt_h[key2];
            if (t + 3 < nt) kb3 = sel_entry(t + 3);
        }
        __builtin_amdgcn_sched_barrier(0);
        // K operands of keys 0..31: in flight while the next tile's loads are set up
        bf16x8 ka[D / 16], kb2[D / 16];
        if constexpr (ACTIVE) read_k<STAGE * TILEB>(ka, kaddr);
        if (t + 1 < nt) issue_loads(meta[(t + 1) % 3], STAGE ^ 1);
        const TileMeta &mt = meta[t % 3];
        if constexpr (ACTIVE) {

        // The score accumulators start from the keys' bias (register v is key row 8(v/4)+4g+v%4 of its half),
        // in units of raw scores, so K Q^T lands on top of it: masking and multiplicity cost no vector instruction.
        f32x16 s_acc[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const f32x4 bv = *(const f32x4 *)(&mt.bias[32 * kb + 8 * q4 + 4 * g]);
#pragma unroll
                for (int e = 0; e < 4; ++e) s_acc[kb][4 * q4 + e] = bv[e];
            }
        wait_k(ka);
        read_k<STAGE * TILEB + 32 * ROWB>(kb2, kaddr);  // keys 32..63, land during the first eight products
#pragma unroll
        for (int s = 0; s < D / 16; ++s) s_acc[0] = mfma_bf16_32x32x16(ka[s], qf[s], s_acc[0]);
        wait_k(kb2);
        // V^T fragments of keys 0..31 of the tile: issued now, they land during the softmax arithmetic
        s16x4 va[2][D / 32][2], vb[2][D / 32][2];
        read_vt<STAGE * TILEB>(va, vaddr);
#pragma unroll
        for (int s = 0; s < D / 16; ++s) s_acc[1] = mfma_bf16_32x32x16(kb2[s], qf[s], s_acc[1]);
        // P = exp2(scale * (S - m_ref)) with a lazily updated reference (any reference cancels in O / l).
        // The row maximum is not taken per tile: P is computed against the reference as it stands and the tile's own
        // row sums tell whether some score ran away from it (a sum beyond 2^15, or an overflow); only then, and
        // while a query has no reference yet, is the maximum taken and O and the sums rescaled.  The reference is
        // always the maximum over some prefix of the keys, so nothing underflows that the exact maximum would keep.
        bf16x2 ones;
        ones[0] = (__bf16)1.0f;
        ones[1] = (__bf16)1.0f;
        bf16x8 pf[2][2];
        float lt0, lt1;
        auto compute_p = [&]() {
            lt0 = 0.0f;
            lt1 = 0.0f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int hh = 0; hh < 2; ++hh) {
                    bf16x2 pr[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float p0 = __builtin_amdgcn_exp2f(fmaf(s_acc[kb][8 * hh + 2 * j], scale_log2, neg_ms));
                        const float p1 = __builtin_amdgcn_exp2f(fmaf(s_acc[kb][8 * hh + 2 * j + 1], scale_log2, neg_ms));
                        pr[j][0] = (__bf16)p0;
                        pr[j][1] = (__bf16)p1;
                        // the sums take the rounded P, the values the PV product sees
                        if (j & 1) lt1 = __builtin_amdgcn_fdot2_f32_bf16(pr[j], ones, lt1, false);
                        else lt0 = __builtin_amdgcn_fdot2_f32_bf16(pr[j], ones, lt0, false);
                    }
                    __builtin_memcpy(&pf[kb][hh], pr, 16);
                }
        };
        bool renew = __any(m_ref == -INFINITY);   // wave-uniform
        if (!renew) {
            compute_p();
            renew = __any(!(lt0 + lt1 <= 32768.0f));
        }
        if (renew) {
            float mx = s_acc[0][0];
#pragma unroll
            for (int v = 1; v < 16; ++v) mx = fmaxf(mx, s_acc[0][v]);
#pragma unroll
            for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s_acc[1][v]);
            mx = fmaxf(mx, shfl_xor(mx, 32));
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
            compute_p();
        }
        l0 += lt0;
        l1 += lt1;

        wait_vt(va);
        read_vt<STAGE * TILEB + 32 * ROWB>(vb, vaddr);  // keys 32..63, land during the first eight products
        pv_mfma(o_acc, va, pf[0]);
        wait_vt(vb);
        pv_mfma(o_acc, vb, pf[1]);
        }

        // row table of tile t+2, second half
        __builtin_amdgcn_sched_barrier(0);
        if (t + 2 < nt && tid < TK) {
            TileMeta &m2 = meta[(t + 2) % 3];
            m2.idx[tid] = key2 >= 0 ? key2 : 0;
            m2.bias[tid] = key2 >= 0 ? (cnt_h ? __log2f((float)cnt2) * inv_scale_log2 : 0.0f) : -INFINITY;
        }
        kb_ahead = kb3;
    };
    if (b * (NW * 32) + wave * 32 < n_q) {   // wave-uniform
        for (int t = t0; t < nt; t += 2) {
            tile_step(t, std::integral_constant<int, 0>{}, std::true_type{});
            if (t + 1 < nt) tile_step(t + 1, std::integral_constant<int, 1>{}, std::true_type{});
        }
    } else {
        for (int t = t0; t < nt; t += 2) {
            tile_step(t, std::integral_constant<int, 0>{}, std::false_type{});
            if (t + 1 < nt) tile_step(t + 1, std::integral_constant<int, 1>{}, std::false_type{});
        }
    }

    const float l_lane = l0 + l1;
    const float l_tot = l_lane + shfl_xor(l_lane, 32);
    if (part) {   // a fragment of the block: everything a later combination needs, as it sits in the registers
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) part[((wave * (D / 32) + db) * 16 + v) * 64 + lane] = o_acc[db][v];
        part[NW * PART_O_FLOATS + wave * 64 + lane] = m_ref;
        part[NW * PART_O_FLOATS + NW * 64 + wave * 64 + lane] = l_tot;
        __syncthreads();   // the tile stages and row tables are free for the next block
        return;
    }
    // epilogue: normalise, transpose through LDS (K stages are free now), store rows coalesced
    const float inv = l_tot > 0.0f ? 1.0f / l_tot : 0.0f;
    __syncthreads();
    constexpr int OSTR = D + 8;  // bf16 elements per staged row (16-byte pad)
    unsigned short *Os = (unsigned short *)lds + (size_t)wave * 32 * OSTR;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            bf16x8 dummy;
            (void)dummy;
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
            const int qi = b * (NW * 32) + wave * 32 + r;
            if (qi < n_q) *(u32x4 *)(O + ((size_t)h * n_q + qi) * D + cc * 8) = *(const u32x4 *)(Os + r * OSTR + cc * 8);
        }
    }
    if (lse && g == 0 && q_idx < n_q)
        lse[(size_t)h * n_q + q_idx] = l_tot > 0.0f ? (m_ref * scale_log2 + __log2f(l_tot)) * LN2 : -INFINITY;
    __syncthreads();   // the staged output rows have been read: the tile stages are free for the next block
}


// One query block per workgroup; two workgroups per CU, started as slots free up.
template <int NW>
__global__ __launch_bounds__(NW * 64, 2) void attn_bf16_d128_kernel(
    const unsigned short *__restrict__ Q, const unsigned short *__restrict__ K, const unsigned short *__restrict__ V,
    const int32_t *__restrict__ cnt, const int32_t *__restrict__ len, const int32_t *__restrict__ sel,
    const int32_t *__restrict__ nsel, int n_q, int C, int bk_shift, int n_sel, int n_qb, int H, float scale_log2, float inv_scale_log2,
    unsigned short *__restrict__ O, float *__restrict__ lse) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    // workgroup -> (head, query block): each XCD (workgroups are dealt round-robin to 8 of them) gets a
    // contiguous range of (head, block) pairs, so neighbouring query blocks share one L2.
    const int total = n_qb * H;
    const int wg = blockIdx.x;
    const int per = (total + 7) / 8;
    const int item = (wg & 7) * per + (wg >> 3);
    if (item >= total) return;
    attend_item<NW>(Q, K, V, cnt, len, sel, nsel, n_q, C, bk_shift, n_sel, n_qb, scale_log2, inv_scale_log2, O, lse, lds,
                    item / n_qb, item % n_qb, 0, INT_MAX, nullptr);
}

// The persistent form (BQ = 128) for the query blocks that whole rounds of one-block workgroups leave over.  The
// (head, block) pairs are dealt to the 8 XCDs in contiguous ranges of `per`, as in the plain kernel; the first `full_per`
// pairs of every range (whole rounds of the workgroups an XCD holds at once) are taken by one workgroup each, and the
// other per - full_per of every range (all of them when full_per is 0) as follows.  Every such query block stands for NT tiles (its list may be shorter), the
// blocks, range after range, make one sequence of tiles, and each of the P resident workgroups takes an equal,
// contiguous share of it: whole blocks are finished in place, a block cut by a share's boundary leaves one fragment per
// share that touches it (slot 0 of a workgroup: a block begun by an earlier workgroup; slot 1: a block it begins but
// does not finish), and attn_combine_kernel puts the fragments together.  However the number of blocks left over
// compares with the number of resident workgroups, every workgroup does the same amount of work.
__global__ __launch_bounds__(256, 2) void attn_bf16_d128_sk_kernel(
    const unsigned short *__restrict__ Q, const unsigned short *__restrict__ K, const unsigned short *__restrict__ V,
    const int32_t *__restrict__ cnt, const int32_t *__restrict__ len, const int32_t *__restrict__ sel,
    const int32_t *__restrict__ nsel, int n_q, int C, int bk_shift, int n_sel, int n_qb, TailMap tm, int n_plain, int NT,
    float scale_log2, float inv_scale_log2, unsigned short *__restrict__ O, float *__restrict__ lse, float *__restrict__ ws) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    // The first 8 * full_per workgroups of the launch are the plain kernel's (range wg & 7, pair wg >> 3 of it, the whole
    // block): one launch, so that the shares start as soon as workgroups of the last whole round finish.
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
            if (t_begin > 0 || t_end < NT) part = ws + ((size_t)i * 2 + (t_begin > 0 ? 0 : 1)) * PART_FLOATS;
            attend_item<4>(Q, K, V, cnt, len, sel, nsel, n_q, C, bk_shift, n_sel, n_qb, scale_log2, inv_scale_log2, O, lse,
                           lds, item / n_qb, item % n_qb, t_begin, t_end, part);
        }
        v = (long long)vi * NT + t_end;
    }
}

// Fragments of the query blocks that attn_bf16_d128_sk_kernel cut: workgroup (i, db) of this launch puts together, for the
// 32 coordinates db of d, the block that share i begins but does not finish (its slot 1, then slot 0 of the following
// shares while they lie inside the block).  Same wavefront / lane layout as the fragments; any reference maximum is as good
// as the true one.  One workgroup per block and quarter of d: the rows of four fragments are in flight together, so a
// block costs one or two memory round trips.
// lse_offset: added to the base-2 logarithm (the 8-bit kernel's probabilities carry a fixed power of two).
__global__ __launch_bounds__(256) void attn_combine_kernel(const float *__restrict__ ws, int P, int n_q, int n_qb, TailMap tm,
                                                           int NT, float scale_log2, float lse_offset,
                                                           unsigned short *__restrict__ O, float *__restrict__ lse) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int i = blockIdx.x, db = blockIdx.y;
    const long long W = tm.tiles(NT);
    const long long start = i * W / P, end = (i + 1) * W / P;
    if (end >= W || end % NT == 0) return;          // share i ends with a whole block
    const int vi = (int)(end / NT);
    if ((long long)vi * NT < start) return;         // the block began in an earlier share: that one combines it
    const int item = tm.item(vi);
    if (item >= tm.total) return;                   // no such block: nothing was written for it
    const long long item_end = (long long)(vi + 1) * NT;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, g = lane >> 5;
    const int h = item / n_qb, b = item % n_qb;
    // fragments: (i, slot 1), then (k, slot 0) for k = i + 1 .. while share k starts inside the block
    int n_frag = 1;
    while (i + n_frag < P && (i + n_frag) * W / P < item_end) ++n_frag;
    auto frag = [&](int f) -> const float * { return ws + ((size_t)(i + f) * 2 + (f == 0 ? 1 : 0)) * PART_FLOATS; };
    float m_all = -INFINITY;
    for (int f = 0; f < n_frag; ++f) m_all = fmaxf(m_all, frag(f)[4 * PART_O_FLOATS + wave * 64 + lane]);
    float o[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) o[v] = 0.0f;
    float l_tot = 0.0f;
    constexpr int FB = 4;   // fragments whose rows are loaded together
    for (int f0 = 0; f0 < n_frag; f0 += FB) {
        float mf[FB], lf[FB], of[FB][16];
#pragma unroll
        for (int u = 0; u < FB; ++u) {
            const float *p = frag(min(f0 + u, n_frag - 1));
            mf[u] = p[4 * PART_O_FLOATS + wave * 64 + lane];
            lf[u] = p[4 * PART_O_FLOATS + 4 * 64 + wave * 64 + lane];
#pragma unroll
            for (int v = 0; v < 16; ++v) of[u][v] = p[((wave * (D / 32) + db) * 16 + v) * 64 + lane];
        }
#pragma unroll
        for (int u = 0; u < FB; ++u) {
            const float w = (f0 + u >= n_frag || mf[u] == -INFINITY) ? 0.0f : __builtin_amdgcn_exp2f((mf[u] - m_all) * scale_log2);
            l_tot += w * lf[u];
#pragma unroll
            for (int v = 0; v < 16; ++v) o[v] += w * of[u][v];
        }
    }
    const float inv = l_tot > 0.0f ? 1.0f / l_tot : 0.0f;
    constexpr int OS = 32 + 8;   // bf16 elements per staged row (this quarter of d, padded)
    unsigned short *Os = (unsigned short *)lds + (size_t)wave * 32 * OS;
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
        typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
        bf16x4 wv;
#pragma unroll
        for (int e = 0; e < 4; ++e) wv[e] = (__bf16)(o[4 * q4 + e] * inv);
        *(bf16x4 *)(Os + col * OS + 8 * q4 + 4 * g) = wv;
    }
    __syncthreads();
    const int rr = lane >> 2, cc = lane & 3;
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int r = it * 16 + rr;
        const int qi = b * 128 + wave * 32 + r;
        if (qi < n_q) *(u32x4 *)(O + ((size_t)h * n_q + qi) * D + 32 * db + cc * 8) = *(const u32x4 *)(Os + r * OS + cc * 8);
    }
    const int q_idx = b * 128 + wave * 32 + col;
    if (db == 0 && lse && g == 0 && q_idx < n_q)
        lse[(size_t)h * n_q + q_idx] = l_tot > 0.0f ? (m_all * scale_log2 + lse_offset + __log2f(l_tot)) * LN2 : -INFINITY;
}

}  // namespace d128

// The combination launch for any kernel that leaves fragments in the layout above (the bf16 and the 8-bit one).
int launch_attn_combine(const void *ws, int n_q, int n_qb, TailMap tm, int NT, float scale_log2, float lse_offset, void *O,
                        float *lse, hipStream_t s) {
    using namespace d128;
    hipLaunchKernelGGL(attn_combine_kernel, dim3(SK_WORKGROUPS, D / 32), dim3(256), 4 * 32 * (32 + 8) * 2, s, (const float *)ws,
                       SK_WORKGROUPS, n_q, n_qb, tm, NT, scale_log2, lse_offset, (unsigned short *)O, lse);
    if (hipGetLastError() != hipSuccess) return FASTAR_ERR_HIP;
    return FASTAR_OK;
}

// more than 64 KiB of LDS per workgroup has to be requested once per kernel and device
int attn_d128_setup() {
    using namespace d128;
    static DeviceOnce once;
    return once.run([](int) {
        if (hipFuncSetAttribute((const void *)attn_bf16_d128_kernel<4>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                LDS_BYTES) != hipSuccess ||
            hipFuncSetAttribute((const void *)attn_bf16_d128_kernel<2>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                LDS_BYTES) != hipSuccess ||
            hipFuncSetAttribute((const void *)attn_bf16_d128_sk_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                LDS_BYTES) != hipSuccess)
            return FASTAR_ERR_HIP;
        return FASTAR_OK;
    });
}

// Launcher used by sparse_attn_fwd for bf16, d = 128.  BQ in {64, 128}.
int launch_attn_bf16_d128(const void *Q, int n_q, const void *K, const void *V, const int32_t *cnt, const int32_t *len,
                          int H, int C, const int32_t *sel, const int32_t *nsel, int BQ, int bk_shift, int n_sel,
                          float scale_log2, void *O, float *lse, hipStream_t s) {
    using namespace d128;
    if (const int rc = attn_d128_setup(); rc != FASTAR_OK) return rc;
    const int n_qb = (n_q + BQ - 1) / BQ;
    const dim3 grid((unsigned)(((n_qb * H + 7) / 8) * 8));
    if (BQ == 128)
        hipLaunchKernelGGL(attn_bf16_d128_kernel<4>, grid, dim3(256), LDS_BYTES, s, (const unsigned short *)Q,
                           (const unsigned short *)K, (const unsigned short *)V, cnt, len, sel, nsel, n_q, C, bk_shift,
                           n_sel, n_qb, H, scale_log2, 1.0f / scale_log2, (unsigned short *)O, lse);
    else
        hipLaunchKernelGGL(attn_bf16_d128_kernel<2>, grid, dim3(128), LDS_BYTES, s, (const unsigned short *)Q,
                           (const unsigned short *)K, (const unsigned short *)V, cnt, len, sel, nsel, n_q, C, bk_shift,
                           n_sel, n_qb, H, scale_log2, 1.0f / scale_log2, (unsigned short *)O, lse);
    if (hipGetLastError() != hipSuccess) return FASTAR_ERR_HIP;
    return FASTAR_OK;
}

// The persistent form of the same attention (BQ = 128): every resident workgroup gets an equal share of the tiles.
// ws: SK_WORKGROUPS * 2 fragments (attn_sk_ws_bytes()).
size_t attn_sk_ws_bytes() { return (size_t)d128::SK_WORKGROUPS * 2 * d128::PART_FLOATS * sizeof(float); }

// full_per: (head, block) pairs per XCD range that the plain kernel takes first, in whole rounds of the 64 workgroups an
// XCD holds (0: the persistent kernel takes everything); the rest of every range goes to the persistent kernel.
int launch_attn_bf16_d128_sk(const void *Q, int n_q, const void *K, const void *V, const int32_t *cnt, const int32_t *len,
                             int H, int C, const int32_t *sel, const int32_t *nsel, int bk_shift, int n_sel,
                             float scale_log2, void *O, float *lse, void *ws, int full_per, hipStream_t s) {
    using namespace d128;
    if (const int rc = attn_d128_setup(); rc != FASTAR_OK) return rc;
    const int n_qb = (n_q + 127) / 128;
    const int NT = (int)((((long long)n_sel << bk_shift) + TK - 1) / TK);
    const TailMap tm = {(n_qb * H + 7) / 8, full_per, n_qb * H};
    if (full_per < 0 || full_per >= tm.per) return FASTAR_ERR_INVALID_ARG;
    const int n_plain = 8 * full_per;
    hipLaunchKernelGGL(attn_bf16_d128_sk_kernel, dim3(n_plain + SK_WORKGROUPS), dim3(256), LDS_BYTES, s, (const unsigned short *)Q,
                       (const unsigned short *)K, (const unsigned short *)V, cnt, len, sel, nsel, n_q, C, bk_shift, n_sel,
                       n_qb, tm, n_plain, NT, scale_log2, 1.0f / scale_log2, (unsigned short *)O, lse, (float *)ws);
    if (hipGetLastError() != hipSuccess) return FASTAR_ERR_HIP;
    return launch_attn_combine(ws, n_q, n_qb, tm, NT, scale_log2, 0.0f, O, lse, s);
}

}  // namespace fastar
