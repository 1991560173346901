/*
 * libfastar: the attention hot path of FAST-AR on one MI355X (gfx950), as a C ABI.
 *
 * Four operations, as the method section of the paper states them, plus the code they share:
 *   fastar_encode        shared low-dimensional 8-bit ANN code of queries / keys / prompt keys
 *   tempcache_compress   merge one frame of new K/V into the bounded per-head cache (TempCache)
 *   ann_select_self      key blocks each query block attends to (AnnSA)
 *   ann_select_cross     prompt tokens each query block attends to (AnnCA)
 *   ann_cross_attn_fwd   the same selection and the attention over it in one launch
 *   sparse_attn_fwd      softmax attention over the selected keys only, with the log-multiplicity bias
 *
 * Conventions (all entry points):
 *   - Every pointer is a DEVICE pointer unless it points to one of the small structs below, which
 *     are read on the host at call time.  The caller owns every buffer; the library allocates
 *     nothing and never synchronises with the host.  It keeps no state that a result depends on: the
 *     only process-wide data are per-device marks that the one-time kernel set-up has been done
 *     (fastar_init, or lazily and thread-safely by the first call that needs it).
 *   - `stream` is a hipStream_t passed as void*.  Work is enqueued on it and the call returns.
 *   - Tensors are DENSE row-major: [H, N, d] means element (h, n, t) at (h*N + n)*d + t; there are no
 *     stride arguments.  The key/value tiles of the attention kernels are fetched straight into LDS
 *     from one base address per tile with fixed row pitch d * sizeof(element), and the cache arrays
 *     K, V, code, cnt, stamp are indexed by one slot number; a strided view would put an address
 *     computation per row back into those loops.  A caller that holds a strided view passes a
 *     contiguous copy.  The batch dimension is folded into H.  Rows of Q/K/V/O must be 16-byte aligned.
 *   - dtype: FASTAR_F32 (float) or FASTAR_BF16 (bfloat16).  Q, K, V, O of one call share it.
 *   - Return value: FASTAR_OK, or a negative code found on the host before anything is launched
 *     (INVALID_ARG: null / negative / inconsistent argument; UNSUPPORTED: a shape the kernels are
 *     not built for; WORKSPACE: workspace too small), or FASTAR_ERR_HIP when a launch failed.
 *     Conditions only the device can see (a full cache dropping tokens) are reported through the
 *     `stats` output, never through the return value.
 *   - Index outputs are deterministic: every decision is taken on exact integer scores with ties
 *     going to the lowest index, so repeated calls and other implementations of the same
 *     definition give identical bits.
 */
#ifndef FASTAR_H
#define FASTAR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FASTAR_OK 0
#define FASTAR_ERR_INVALID_ARG (-1)
#define FASTAR_ERR_UNSUPPORTED (-2)
#define FASTAR_ERR_WORKSPACE (-3)
#define FASTAR_ERR_HIP (-4)
#define FASTAR_ERR_STATIC_SCRATCH (-5) /* the problem needs more than FASTAR_STATIC_SCRATCH_BYTES */

/* size of the library's static device scratch (ann_select_self_static), held by every GPU the library runs on */
#define FASTAR_STATIC_SCRATCH_BYTES (32 * 1024 * 1024)

#define FASTAR_F32 0
#define FASTAR_BF16 1

#define FASTAR_OP_COMPRESS 1
#define FASTAR_OP_SELECT_SELF 2
#define FASTAR_OP_SELECT_CROSS 3
#define FASTAR_OP_SELECT_LSH 4
#define FASTAR_OP_SELECT_BUCKETS 5 /* pass the number of prompt tokens as r */
#define FASTAR_OP_ATTN 6           /* sparse_attn_fwd_ws, sparse_attn_fwd_fp8_ws: a fixed amount, whatever the shape */

/* representative key of a merged TempCache group (tempcache_compress, rep_mode) */
#define FASTAR_REP_LAST 0
#define FASTAR_REP_MEAN 1
#define FASTAR_REP_MEDOID 2

/*
 * Bounded per-head KV cache with multiplicities (Lemma 1 of the paper: a group of merged keys is
 * kept as one representative key, the mean of the group's values and the group size m, which
 * enters attention as a +log m logit shift).  Capacity C slots per head, len[h] <= C of them live.
 */
typedef struct {
    void *K;        /* [H,C,d] dtype   representative = most recent key of each group            */
    void *V;        /* [H,C,d] dtype   mean value of each group                                  */
    int8_t *code;   /* [H,C,r]         ANN code of K                                             */
    int32_t *cnt;   /* [H,C]           multiplicity m >= 1 of live slots                         */
    int32_t *stamp; /* [H,C]           frame id of the slot's last refresh                       */
    int32_t *len;   /* [H]             live slots                                                */
    int32_t H, C, d, r, dtype;
} fastar_cache;

/*
 * Definition of the ANN code (Sec. 5.1: shared low-dimensional random projection + low-bit
 * quantisation, 8 bit by default), in integer arithmetic so that every score is exact:
 *   xq[t] = clamp(rint(x[t] * qscale), -127, 127)           one float32 multiply, ties to even
 *   y[j]  = sum_t R[t][j] * xq[t]                           int32
 *   c[j]  = clamp(floor((y[j] + 2^(shift-1)) / 2^shift), -127, 127)
 */
typedef struct {
    const int8_t *R; /* [d,r] device, entries -1 / +1 */
    float qscale;
    int32_t shift;   /* >= 1 */
} fastar_codec;

/*
 * One-time set-up for the CURRENT device: lets the kernels that stage large tiles use more than 64 KB of LDS.
 * Optional: every entry point does the part it needs on its first call on a device (thread-safe).  Call it before
 * capturing entry points into a HIP graph, so that no attribute call falls inside the capture.  Launches nothing.
 */
int fastar_init(void);

/* Library version string (host pointer, static storage). */
const char *fastar_version(void);

/* Human-readable name of a return code (host pointer, static storage). */
const char *fastar_strerror(int code);

/*
 * Bytes of device workspace an operation needs (FASTAR_OP_*).  Arguments that an operation does
 * not use are ignored.  COMPRESS: H, C, n_new (as n_q), r.  SELECT_SELF: H, n_q, C (as n_k), BQ,
 * BK, n_rep, r.  SELECT_CROSS: H, n_q, n_p (as n_k), BQ.  SELECT_LSH: H, n_q, C (as n_k), n_bits (as r), BQ, BK,
 * n_rep.  Returns 0 for an unknown op.
 */
size_t fastar_workspace_bytes(int op, int H, int n_q, int n_k, int r, int BQ, int BK, int n_rep);

/*
 * ANN codes (Sec. 5.1) of n_vec vectors.
 *   x        [n_vec, d] dtype (device), d in {64, 128}
 *   codec    host struct; codec->R device [d, r], r in {32, 64}
 *   code_out [n_vec, r] int8 (device)
 */
int fastar_encode(const void *x, int dtype, int64_t n_vec, int d, const fastar_codec *codec, int r,
                  int8_t *code_out, void *stream);

/*
 * Prompt-induced buckets (Sec. 5.4, first paragraph: self-attention reuses the semantic buckets found by
 * cross-attention pruning; a query is assigned to one or more buckets and attends only to keys of the same
 * bucket(s)).  The prompt tokens are the buckets: a code belongs to the m prompt tokens with the largest code inner
 * product (the products ann_select_cross ranks prompt tokens by), ties to the smaller token id.
 *   code   [H,C,r] int8 (device), pcode [H,n_p,r] int8 (device), both 16-byte aligned
 *   idx    [H,n] int32 rows to assign (device; entries < 0 or >= C are skipped, repeats are harmless), or NULL for
 *          rows 0..n-1 (n <= C): a caller that keeps one bucket row per cache slot re-assigns only the slots
 *          tempcache_compress wrote (its merge_map)
 *   bucket [H,C,m] int32 out (device): token ids, best first; -1 where n_p < m; rows not named are left as they are
 * Supported: r in {32, 64}, n_p <= 2048, m <= 8.
 */
int ann_prompt_buckets(const int8_t *code, int C, const int32_t *idx, int n, const int8_t *pcode, int n_p, int H, int r,
                       int m, int32_t *bucket, void *stream);

/*
 * AnnSA on those buckets: a query block owns the buckets of its queries, a key block those of its live keys; a key
 * block is a candidate only if the two share a bucket; of the candidates the n_sel that share the most are kept
 * (ties: lowest index), written ascending to sel, -1 padded; nsel = their number (it can be 0).  The first n_sink and
 * the last n_local live key blocks are always kept and count against the budget (n_sink + n_local <= n_sel).
 *   qbucket [H,n_q,m], kbucket [H,C,m] int32 (entries outside [0, n_p) are ignored), len [H];
 *   sel [H,n_qb,n_sel], nsel [H,n_qb] out;  ws of fastar_workspace_bytes(FASTAR_OP_SELECT_BUCKETS, H, n_q, C, n_p, BQ, BK, 0).
 * Supported: n_p <= 2048; ceil(n_q/BQ) * ceil(n_p/32) * 4 bytes <= 48 KiB.
 */
int ann_select_buckets(const int32_t *qbucket, int n_q, const int32_t *kbucket, const int32_t *len, int H, int C, int m,
                       int n_p, int BQ, int BK, int n_sel, int n_sink, int n_local, int32_t *sel, int32_t *nsel, void *ws,
                       size_t ws_bytes, void *stream);

/*
 * Codes that are really `bits` wide (appendix, "Quantization precision for ANN matching": the bit width of the
 * retrieval codes is varied; narrower codes are cheaper to store and to stream).  As fastar_encode, but the last step
 * saturates to +-(2^(bits-1) - 1) and entry j of a vector occupies bits [bits*(j mod 8/bits), +bits) of byte
 * j / (8/bits): packed_out [n_vec, r*bits/8] uint8 (device, 4-byte aligned).  bits in {2, 4, 8}; 8 is fastar_encode.
 * Supported for bits < 8: r = 32.
 */
int fastar_encode_packed(const void *x, int dtype, int64_t n_vec, int d, const fastar_codec *codec, int r, int bits,
                         uint8_t *packed_out, void *stream);

/*
 * ann_select_self_forced on such packed codes: qcode [H,n_q,r*bits/8], kcode [H,C,r*bits/8]; the result is that of
 * ann_select_self_forced on the unpacked entries.  The key codes are streamed as they are stored (r*bits/8 bytes per
 * key) and widened in registers.  Same workspace as ann_select_self (the summaries are kept one byte per entry).
 * Supported for bits < 8: r = 32.
 */
int ann_select_self_packed(const int8_t *qcode, int n_q, const int8_t *kcode, const int32_t *len, int H, int C, int r,
                           int bits, int BQ, int n_rep, int BK, int n_sel, int n_sink, int n_local, int32_t *sel,
                           int32_t *nsel, void *ws, size_t ws_bytes, void *stream);

/*
 * Sign codes, the hash of the LSH paragraph of Sec. 5.1: one bit per random projection, the side of the
 * hyperplane the quantised vector lies on.  bit j = 1 iff sum_t R[t][j] * xq[t] >= 0, xq as in fastar_codec.
 *   x        [n_vec, d] dtype (device), d in {64, 128}
 *   R        [d, n_bits] int8 entries -1 / +1 (device), n_bits in {64, 128, 256}
 *   bits_out [n_vec, n_bits/32] uint32 (device); bit j of a vector sits in word j/32 at position j%32
 */
int fastar_encode_sign(const void *x, int dtype, int64_t n_vec, int d, const int8_t *R, float qscale, int n_bits,
                       uint32_t *bits_out, void *stream);

/*
 * Selection on sign codes (Sec. 5.3 / 5.4 with the LSH family of Sec. 5.1): candidates are ranked by the number of
 * hash bits they share with the query side.  Query block b (BQ queries) is summarised by n_rep majority codes, one
 * per run of BQ/n_rep queries (bit j = 1 iff at least half of the run's queries have it set); the score of key
 * block kb (BK keys) is the largest number of equal bits between a summary and a live key of the block; the
 * min(n_sel, ceil(len/BK)) best key blocks (ties: lowest index) are written ascending to sel, -1 padded.
 * n_rep = BQ, BK = 1 is the cross-attention form (a prompt token is scored by its best-matching query).
 *   qbits [H,n_q,W], kbits [H,C,W] uint32 (W = n_bits/32), len [H];  sel [H,n_qb,n_sel], nsel [H,n_qb] out.
 * Supported: n_bits in {64,128,256}; BK a power of two <= 64 or a multiple of 64; BQ a multiple of n_rep.
 */
int ann_select_lsh(const uint32_t *qbits, int n_q, const uint32_t *kbits, const int32_t *len, int H, int C,
                   int n_bits, int BQ, int n_rep, int BK, int n_sel, int32_t *sel, int32_t *nsel, void *ws,
                   size_t ws_bytes, void *stream);

/*
 * Hash-table form of ann_select_lsh (Sec. 5.1, LSH paragraph: a query only compares against keys that land in the same
 * bucket(s); Sec. 2: multi-table bucket probing).  The hash bits are cut into n_bits / band_bits bands, one table each;
 * a vector's bucket in a table is its band.  A summary and a key collide in a table when their buckets differ in at
 * most `radius` bits (0: the same bucket; more: the neighbouring buckets are probed as well).  A pair scores its
 * colliding tables, a key block its best (summary, live key) pair; key blocks without a collision are no candidates;
 * of the candidates the n_sel best are kept (ties: lowest index), -1 padded; nsel = their number (it can be 0).  The
 * first n_sink / last n_local live key blocks are always kept (n_sink + n_local <= n_sel).
 * Same arrays and workspace as ann_select_lsh.  Supported: band_bits in {4, 8, 16, 32}.
 */
int ann_select_lsh_buckets(const uint32_t *qbits, int n_q, const uint32_t *kbits, const int32_t *len, int H, int C,
                           int n_bits, int band_bits, int radius, int BQ, int n_rep, int BK, int n_sel, int n_sink,
                           int n_local, int32_t *sel, int32_t *nsel, void *ws, size_t ws_bytes, void *stream);

/*
 * TempCache (Sec. 5.2 and Lemma 1): merge one frame of n_new tokens per head into the cache.  Every
 * decision is taken against the cache as it is at entry; a chunk of several frames is several calls.
 *   1. probe code cp_i = code(P_new[i]) (P_new NULL => K_new), key code ck_i = code(K_new[i]).
 *   2. top-1 match among the candidate slots (cand [H,n_cand] names a SET of slot ids: its order and
 *      repeated ids mean nothing, ids outside [0,len) are skipped; cand NULL => every live slot):
 *      j*(i) = argmax_j S(i,j), ties to the smallest slot,
 *      S = 2 cp_i.code_j - |code_j|^2 (metric 0, nearest in code space) or cp_i.code_j (metric 1).
 *   3. similarity threshold on the 8-bit quantised full-width keys a = xq(K_new[i]), b = xq(K[j*]):
 *      merged_i <=> a.b > 0 and (a.b)^2 * 65536 >= tau2_q16 * |a|^2 |b|^2, with
 *      tau2_q16 = rint(tau^2 * 65536) in [0, 131072].
 *   4. every slot keeps, of the tokens merged into it, the one closest in code space (metric 0:
 *      S - |cp_i|^2, metric 1: S; ties to the smallest token) as its new representative key; its
 *      value becomes the mean over the enlarged group and its multiplicity grows by the joiners.
 *      rep_mode FASTAR_REP_MEAN (appendix ablation "Representative selection in KV merging") stores the
 *      multiplicity-weighted mean key instead: float32, multiplicity * old key, then the joiners' keys in
 *      ascending token order, one division, one rounding to dtype; the slot's code is the code of the
 *      stored key (one more launch).  FASTAR_REP_MEDOID stores the medoid key: of the slot's stored key (standing for
 *      the multiplicity tokens merged so far) and this call's joiners (weight 1 each) the one with the smallest weighted
 *      total squared distance to the others in code space (exact integers; ties to the stored key, then the smaller
 *      token); the stored key winning leaves key and code as they are.  FASTAR_REP_LAST is the method's own choice and
 *      the fast path.
 *   5. unmerged tokens are appended in token order.  If the cache would exceed C, the live slots
 *      that received no token in this call are evicted, smallest (stamp, slot) first, and refilled
 *      in ascending slot order; if there are too few of those, the last unmerged tokens are dropped.
 *   K_new, V_new, P_new [H,n_new,d] dtype;  frame_id is stored as the stamp of every written slot.
 * Outputs:
 *   merge_map [H,n_new] int32  destination slot of each token, -1 if dropped
 *   merged    [H,n_new] uint8  1 if the token joined an existing slot
 *   stats     [H,8]     int32  {len after, n_merged, n_appended, n_evicted, n_dropped, 0, 0, status}
 *                              status 0; 1 if a bounded wait inside the eviction plan ran out (its workgroups, which
 *                              meet through global memory, were not all running at once): nothing of this call is
 *                              applied to the head then, its K, V, code, cnt, stamp and len stay as they were, every
 *                              token of the head is reported dropped (merge_map -1, merged 0, n_dropped = n_new), and a
 *                              persistent workspace has to be zero-filled again before its next use; 2 if the stamps
 *                              of the evictable slots span 2^20 frames or more: the choice of victims is then not
 *                              guaranteed to be the oldest-first one
 *                              3 if ws_persistent was set for a workspace that is neither zero-filled nor left by
 *                              a finished call: nothing is applied either (as for status 1)
 *   ws / ws_bytes              workspace of fastar_workspace_bytes(FASTAR_OP_COMPRESS, ...), 256-byte aligned
 *   ws_persistent              0: the workspace may hold anything (the call clears what it needs: one launch more).
 *                              1: the caller zero-filled the workspace once and since then only calls of this
 *                              function on this cache have written to it; every call leaves it as clean as a
 *                              zero-filled one, so the match can go straight on to the threshold test (for candidate
 *                              lists that fit LDS with P_new NULL; other calls ignore the flag).  The library still
 *                              keeps no state of its own: the state is the caller's buffer.
 * The cache struct and the codec struct are host structs; cache->len is updated on the device.
 * Supported: d in {64,128}, r in {32,64}; C up to about 393 000 * min(16, 1024 / H) slots per head (the eviction
 *            plan runs on that many workgroups per head and each keeps a bitmap of its share of the slots in LDS):
 *            6 million for up to 64 heads; FASTAR_ERR_UNSUPPORTED otherwise.
 */
int tempcache_compress(const fastar_cache *cache, const fastar_codec *codec, const void *K_new,
                       const void *V_new, const void *P_new, int n_new, const int32_t *cand, int n_cand,
                       int metric, int32_t tau2_q16, int32_t frame_id, int rep_mode, int32_t *merge_map,
                       uint8_t *merged, int32_t *stats, void *ws, size_t ws_bytes, int ws_persistent, void *stream);

/*
 * AnnSA (Sec. 5.4 with the ANN goal of Sec. 5.1): for every head and every block of BQ queries,
 * the n_out = min(n_sel, ceil(len/BK)) key blocks of BK keys with the largest code score.
 *   Query block b is summarised by n_rep mean codes, one per run of g = BQ/n_rep queries:
 *   rep = floor((sum of the run's codes + floor(g/2)) / g); runs without a query are skipped.
 *   Score of key block kb = max over summaries and over the block's live keys k < len of rep.code_k.
 *   Ties go to the smaller block index; the result is written in ascending block order.
 *   qcode [H,n_q,r], kcode [H,C,r], len [H]
 *   sel   [H,n_qb,n_sel] int32 out, padded with -1;  nsel [H,n_qb] int32 out;  n_qb = ceil(n_q/BQ)
 * Supported: r in {32,64}; BQ a multiple of n_rep; n_rep in {1,2,4,8,16,32}; BK a multiple of 32;
 *            at most 1024 query blocks per head.
 */
int ann_select_self(const int8_t *qcode, int n_q, const int8_t *kcode, const int32_t *len, int H, int C, int r,
                    int BQ, int n_rep, int BK, int n_sel, int32_t *sel, int32_t *nsel, void *ws,
                    size_t ws_bytes, void *stream);

/*
 * AnnSA with forced key blocks (Sec. 2: rolling-window generators keep their first frames as an attention sink; a
 * local window is the usual companion): as ann_select_self, but the first n_sink key blocks and the last n_local live
 * key blocks of every head are always among the selected ones.  They count against the budget
 * (n_sink + n_local <= n_sel, FASTAR_ERR_INVALID_ARG otherwise); the rest of it goes to the best-scoring other blocks.
 * n_sink = n_local = 0 is ann_select_self.  Same workspace.
 */
int ann_select_self_forced(const int8_t *qcode, int n_q, const int8_t *kcode, const int32_t *len, int H, int C, int r,
                           int BQ, int n_rep, int BK, int n_sel, int n_sink, int n_local, int32_t *sel, int32_t *nsel,
                           void *ws, size_t ws_bytes, void *stream);

/*
 * ann_select_self for callers that cannot allocate or bring a workspace: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and bit-identical outputs as ann_select_self,
 * but the summaries and the score rows live in a static device array of FASTAR_STATIC_SCRATCH_BYTES inside the library
 * (each GPU holds its own copy until the process ends; its address is looked up once per device, by fastar_init or by
 * the first call).  The call allocates nothing: no hipMalloc / hipFree, no workspace argument.
 *   - Problems that need more scratch than that (fastar_workspace_bytes(FASTAR_OP_SELECT_SELF, ...) is the amount;
 *     the world-model layer with 40 heads x 29 query blocks x 3600 key blocks needs 16.8 MB) return
 *     FASTAR_ERR_STATIC_SCRATCH and launch nothing.
 *   - All calls on one GPU share the one array: calls that may overlap on a GPU (different streams, different host
 *     threads) race on it.  Calls on one stream are ordered and safe.  Nothing in the array has to start from zero
 *     and nothing of a previous call is read.
 */
int ann_select_self_static(const int8_t *qcode, int n_q, const int8_t *kcode, const int32_t *len, int H, int C, int r,
                           int BQ, int n_rep, int BK, int n_sel, int32_t *sel, int32_t *nsel, void *stream);

/*
 * AnnCA (Sec. 5.3): for every head and every block of BQ queries, the min(n_sel, n_p) prompt tokens
 * with the largest max over the block's queries of c_q.c_p (a token is kept when at least one query
 * of the block is its neighbour).  Ties to the smaller token index, ascending output, -1 padding.
 *   qcode [H,n_q,r], pcode [H,n_p,r];  sel [H,n_qb,n_sel], nsel [H,n_qb] out.
 * BQ is free (it need not be sparse_attn_fwd's block size): BQ = tokens per frame gives the per-frame selection
 * of Sec. 5.3, whose list the caller then shares among the query blocks of that frame's attention call.
 * Supported: r in {32,64}; n_p <= 12288 (the scores of one query block over the prompt live in LDS).
 */
int ann_select_cross(const int8_t *qcode, int n_q, const int8_t *pcode, int n_p, int H, int r, int BQ,
                     int n_sel, int32_t *sel, int32_t *nsel, void *ws, size_t ws_bytes, void *stream);

/*
 * AnnCA in one launch (Sec. 5.3): the selection of ann_select_cross followed by the attention of sparse_attn_fwd
 * over it (BK = 1, no multiplicities, every prompt token live), for callers that need both and no lse:
 *   sel, nsel  exactly what ann_select_cross(qcode, pcode, BQ, n_sel) writes;
 *   O          exactly what sparse_attn_fwd(Q, Kp, Vp, NULL, len = n_p, sel, nsel, BQ, 1, n_sel, scale) computes
 *              (same arithmetic: bf16 products, fp32 softmax over the selected tokens in one piece).
 *   Q [H,n_q,d], Kp, Vp [H,n_p,d] bf16;  qcode [H,n_q,r], pcode [H,n_p,r];  O [H,n_q,d] bf16 out.
 * Supported: bf16, d = 128, BQ = 128, n_sel <= 64, r in {32,64}, n_p <= 12288; anything else is
 * FASTAR_ERR_UNSUPPORTED and the two separate calls do the same work.  No workspace.
 */
int ann_cross_attn_fwd(const void *Q, const int8_t *qcode, int n_q, const void *Kp, const void *Vp,
                       const int8_t *pcode, int n_p, int H, int d, int dtype, int r, int BQ, int n_sel, float scale,
                       int32_t *sel, int32_t *nsel, void *O, void *stream);

/*
 * Block-sparse attention (Eq. 1 restricted to the candidate set of Sec. 5.1, logits shifted by
 * +ln(cnt) as in Lemma 1).  For query i of query block b, over the live keys J of the key blocks
 * sel[h][b][0 .. nsel[h][b]):  l_j = scale * q_i.k_j + ln(cnt_j);  o_i = sum_j softmax(l)_j v_j;
 * lse_i = ln sum_j exp(l_j).  J empty => o_i = 0, lse_i = -inf.
 *   Q [H,n_q,d], K,V [H,C,d] dtype;  cnt [H,C] or NULL (no bias);  len [H];
 *   sel [H,n_qb,n_sel] (entries < 0 are padding), nsel [H,n_qb];
 *   O [H,n_q,d] dtype out;  lse [H,n_q] float out or NULL.
 * Supported: bf16 with d in {64,128}, BQ in {64,128}, BK a power of two <= 64 (MFMA path, fp32
 * softmax and accumulation); fp32 with d in {64,128}, BQ <= 128, BK <= 64 (plain fp32 arithmetic).
 * scale must be positive and finite (FASTAR_ERR_INVALID_ARG otherwise).  bf16: tile rows are addressed by 32-bit
 * byte offsets inside a head, so C * d * 2 must stay below 2^32 (FASTAR_ERR_UNSUPPORTED otherwise).
 */
int sparse_attn_fwd(const void *Q, int n_q, const void *K, const void *V, const int32_t *cnt,
                    const int32_t *len, int H, int C, int d, int dtype, const int32_t *sel, const int32_t *nsel,
                    int BQ, int BK, int n_sel, float scale, void *O, float *lse, void *stream);

/*
 * sparse_attn_fwd with a workspace: same arguments, same result (to the tolerance of the attention itself: a block
 * that several workgroups share is put together from their partial sums).  With more query blocks than the chip holds
 * at once, in a number that would leave a short last round of workgroups (bf16, d = 128, BQ = 128; the rule is in
 * attention.hip), the launch is split: whole rounds of query blocks are taken by one workgroup each, the blocks left
 * over are cut into equal shares of their tiles for all resident workgroups, blocks cut by a share's boundary leave
 * fragments in `ws`, and a second small launch combines them.  Other shapes run exactly as sparse_attn_fwd and leave
 * `ws` untouched.
 *   ws / ws_bytes  fastar_workspace_bytes(FASTAR_OP_ATTN, ...) bytes, 256-byte aligned; contents need not be kept
 */
int sparse_attn_fwd_ws(const void *Q, int n_q, const void *K, const void *V, const int32_t *cnt, const int32_t *len,
                       int H, int C, int d, int dtype, const int32_t *sel, const int32_t *nsel, int BQ, int BK, int n_sel,
                       float scale, void *O, float *lse, void *ws, size_t ws_bytes, void *stream);

/*
 * 8-bit floating-point K/V for the attention itself (Sec. 5.1, quantised-search paragraph; appendix ablation
 * "Quantization precision for ANN matching" carried over from the retrieval codes to the attended keys and values).
 * Format: E4M3 (OCP 8-bit floating point, "FN": bias 7, subnormals, no infinities, largest finite value 448); values
 * beyond +-448 saturate; conversion rounds to nearest, ties to even.
 *
 * fastar_kv_to_fp8 keeps an 8-bit copy of a bf16 / fp32 cache (d = 128) up to date:
 *   K8   [H, Cp, 128] uint8      codes of the keys, rows as in cache->K; Cp = C rounded up to a multiple of 64
 *   V8T  [H, Cp/64, 128, 64]     codes of the values, every block of 64 slots transposed:
 *                                element (h, blk, t, j) = code of V[h][64 blk + j][t]
 * Every block of 64 slots that holds a live slot with stamp >= stamp_lo is rewritten whole (live slots with the codes
 * of the stored rows, dead slots with zero); other blocks are not touched.  After tempcache_compress(frame_id = f),
 * stamp_lo = f brings the copy up to date; stamp_lo = INT32_MIN rebuilds it.  The caller zero-fills K8 and V8T once:
 * the attention reads whole blocks and a dead slot must hold a finite code.
 */
int fastar_kv_to_fp8(const fastar_cache *cache, int32_t stamp_lo, uint8_t *K8, uint8_t *V8T, void *stream);

/*
 * sparse_attn_fwd over that copy: the same definition (Eq. 1 restricted to the selected key blocks, +ln(cnt) bias of
 * Lemma 1) on the exact values of the E4M3 codes of K and V and of Q rounded to E4M3.  Both products run on the 8-bit
 * floating-point matrix instructions (fp32 accumulation); the softmax weights are rounded to E4M3 before the second
 * product and the row sums are taken over the rounded weights, so every output is a convex combination of the stored
 * values.  Q, O [H,n_q,128] bf16; cnt [H,C] or NULL; len [H]; sel / nsel as for sparse_attn_fwd; lse [H,n_q] or NULL.
 * Supported: d = 128, BQ = 128, BK = 64 (one selection entry = one block of the copy); FASTAR_ERR_UNSUPPORTED otherwise.
 */
int sparse_attn_fwd_fp8(const void *Q, int n_q, const uint8_t *K8, const uint8_t *V8T, const int32_t *cnt,
                        const int32_t *len, int H, int C, int d, const int32_t *sel, const int32_t *nsel, int BQ, int BK,
                        int n_sel, float scale, void *O, float *lse, void *stream);

/*
 * sparse_attn_fwd_fp8 with a workspace, as sparse_attn_fwd_ws is to sparse_attn_fwd: same arguments, same result (to the
 * tolerance of the attention itself); a launch that would end in a short last round of workgroups is split, the query
 * blocks left over are cut into equal shares of their tiles, and a second small launch combines the fragments.  Other
 * shapes run exactly as sparse_attn_fwd_fp8 and leave `ws` untouched.
 *   ws / ws_bytes  fastar_workspace_bytes(FASTAR_OP_ATTN, ...) bytes, 256-byte aligned; contents need not be kept
 */
int sparse_attn_fwd_fp8_ws(const void *Q, int n_q, const uint8_t *K8, const uint8_t *V8T, const int32_t *cnt,
                           const int32_t *len, int H, int C, int d, const int32_t *sel, const int32_t *nsel, int BQ,
                           int BK, int n_sel, float scale, void *O, float *lse, void *ws, size_t ws_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* FASTAR_H */
