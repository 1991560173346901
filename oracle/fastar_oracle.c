/*
 * CPU oracle for the FAST-AR attention hot path.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, step-by-step C.  fp64 accumulation for every floating-point result that is compared
 * with a tolerance (attention outputs, lse, the running mean value), integer arithmetic for every
 * decision.  One exception, by definition and not by accumulation error: the mean-key representative
 * (rep_mode 1).  A stored mean key is re-quantised and re-encoded, so its bits decide later integers
 * (codes, matches, the cosine test); its arithmetic is therefore part of the definition: IEEE float32,
 * multiplicity * old key first, then the joiners' keys in ascending token order, one division, one
 * rounding to the storage type.  tests/test_oracle_tempcache.py pins that order with values on which a
 * float64 accumulation, or another order of the additions, gives different stored bits.
 * Nothing here is shared with the GPU
 * library: no common header, helper, table or constant.  Only tests, the smoke
 * check and the bench's cpu_baseline leg may call it.
 *
 * What each function follows:
 *   oracle_encode              Sec. 5.1 "Attention as approximate nearest neighbour search":
 *                              shared low-dimensional random projection (LSH paragraph) of
 *                              low-bit quantised vectors (quantised-search paragraph, 8 bit).
 *   oracle_encode_packed,      the same codes at 2 or 4 bits per entry, packed (appendix ablation "Quantization precision
 *   oracle_unpack_codes        for ANN matching"); selection on them is oracle_ann_select_self on the unpacked entries.
 *   oracle_tempcache_compress  Sec. 5.2 "KV cache compression using temporal correspondence":
 *                              top-1 neighbour of every new token among cached keys, merge when
 *                              the key similarity passes a threshold, keep the most recent key,
 *                              mean value and multiplicity (Lemma 1; appendix Eqs. for the group
 *                              mean value and the biased logit); rep_mode 1 keeps the mean key instead
 *                              (appendix ablation "Representative selection in KV merging").
 *   oracle_ann_select_self     Sec. 5.4 (AnnSA): keys a query block attends to, ranked by code score.
 *   oracle_ann_select_cross    Sec. 5.3 (AnnCA): prompt tokens with a neighbouring query in the block.
 *   oracle_prompt_buckets,     Sec. 5.4, first paragraph: self-attention restricted to the semantic buckets found by
 *   oracle_ann_select_buckets  cross-attention pruning; the prompt tokens are the buckets, a code belongs to its nearest ones.
 *   oracle_encode_sign         Sec. 5.1, LSH paragraph: one hash bit per random projection (its sign).
 *   oracle_ann_select_lsh      Sec. 5.3 / 5.4 on those hash codes: candidates ranked by the number of hash
 *                              bits they share with the query side (AnnSA with key blocks, AnnCA with BK = 1).
 *   oracle_ann_select_lsh_buckets  the same with hash tables: the code cut into bands, a pair scored by the tables in which
 *                              it falls into the same (or, multi-probe, a neighbouring) bucket; blocks without a collision
 *                              are no candidates (Sec. 5.1 LSH paragraph "same bucket(s)"; Sec. 2 multi-table probing).
 *   oracle_sparse_attn_fwd     Eq. (1) restricted to the candidate set (Sec. 5.1 display), with the
 *                              +log m_t logit shift of Lemma 1.
 *   oracle_recall_density      attention recall / density as defined in the Metrics paragraph.
 *   oracle_fp8_encode/decode,  Sec. 5.1, quantised-search paragraph and the appendix ablation "Quantization precision for
 *   oracle_kv_to_fp8,          ANN matching" name low-bit storage of keys; here the 8-bit floating-point format E4M3
 *   oracle_sparse_attn_fwd_fp8 (OCP "FN": 4 exponent bits, bias 7, 3 mantissa bits, no infinities, largest finite 448) is
 *                              the storage of K and V for the attention itself: the same attention on the exact
 *                              values of the quantised keys, values and queries.
 *
 * Parity pins (tests/test_oracle_*.py): dense softmax attention written independently in
 * numpy, Lemma 1 on exact duplicates, brute-force nearest neighbours and top-k, closed-form
 * code values, identity merge, monotonicity in the threshold, a hand-computed mean key and its
 * coincidence with the last key on exact duplicates; for the sign codes a worked example,
 * sign-flip and scaling invariances, the 1 - angle/pi law of random hyperplanes, brute force in Python.  The eviction policy of
 * oracle_tempcache_compress (what to do when the bounded cache is full) is not in the paper:
 * it is checked by invariants only and is "parity unpinned".
 *
 * dtype: 0 = float32, 1 = bfloat16 stored as uint16 bit patterns.
 * All arrays are dense row-major with the shapes given at each function.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ storage helpers */

static float load_f32(const void *p, int dtype, int64_t idx) {
    if (dtype == 0) return ((const float *)p)[idx];
    uint32_t u = ((uint32_t)((const uint16_t *)p)[idx]) << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

static uint16_t f32_to_bf16(float f) { /* nearest, ties to even */
    uint32_t u;
    memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

static void store_val(void *p, int dtype, int64_t idx, double v) {
    if (dtype == 0)
        ((float *)p)[idx] = (float)v;
    else
        ((uint16_t *)p)[idx] = f32_to_bf16((float)v);
}

static void copy_row(void *dst, int64_t drow, const void *src, int64_t srow, int d, int dtype) {
    size_t es = dtype == 0 ? 4 : 2;
    memcpy((char *)dst + (size_t)drow * d * es, (const char *)src + (size_t)srow * d * es, (size_t)d * es);
}

static int64_t floor_div(int64_t a, int64_t b) { /* b > 0 */
    int64_t q = a / b;
    if (a % b != 0 && a < 0) q -= 1;
    return q;
}

static int clampi(int64_t v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : (int)v); }

/* ------------------------------------------------------------------ encode */

/* Quantise one coordinate to 8 bits: one float32 multiply, round half to even, saturate. */
static int quant8(float x, float qscale) {
    volatile float prod = x * qscale; /* volatile: exactly one IEEE single-precision product */
    float q = rintf(prod);
    if (q > 127.0f) q = 127.0f;
    if (q < -127.0f) q = -127.0f;
    return (int)q;
}

/* Code of one vector: quantise, project on the +-1 matrix R[d][r], shift down with rounding, saturate. */
static void encode_vec(const void *x, int dtype, int64_t base, int d, const int8_t *R, int r, float qscale,
                       int shift, int8_t *code) {
    for (int j = 0; j < r; ++j) {
        int64_t y = 0;
        for (int t = 0; t < d; ++t) y += (int64_t)R[(int64_t)t * r + j] * quant8(load_f32(x, dtype, base + t), qscale);
        int64_t c = floor_div(y + ((int64_t)1 << (shift - 1)), (int64_t)1 << shift);
        code[j] = (int8_t)clampi(c, -127, 127);
    }
}

/* x [n_vec, d] -> code [n_vec, r] */
int oracle_encode(const void *x, int dtype, int64_t n_vec, int d, const int8_t *R, int r, float qscale, int shift,
                  int8_t *code) {
    if (!x || !R || !code || d <= 0 || r <= 0 || shift < 1) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t v = 0; v < n_vec; ++v) encode_vec(x, dtype, v * d, d, R, r, qscale, shift, code + v * r);
    return 0;
}

/*
 * Codes that are really `bits` wide (appendix, "Quantization precision for ANN matching": the retrieval codes' bit
 * width is varied; narrower codes are cheaper to store and to stream).  Same projection; the last step saturates to
 * the range of a `bits`-bit two's complement number without its most negative value, +-(2^(bits-1) - 1), and entry j
 * of a vector occupies bits [bits*(j mod 8/bits), +bits) of byte j / (8/bits).  bits in {2, 4, 8}; 8 is oracle_encode.
 * x [n_vec, d] -> packed [n_vec, r*bits/8] bytes.
 */
int oracle_encode_packed(const void *x, int dtype, int64_t n_vec, int d, const int8_t *R, int r, float qscale,
                         int shift, int bits, uint8_t *packed) {
    if (!x || !R || !packed || d <= 0 || r <= 0 || shift < 1) return -1;
    if ((bits != 2 && bits != 4 && bits != 8) || (r * bits) % 8 != 0) return -1;
    const int lim = (1 << (bits - 1)) - 1, per = 8 / bits;
    const int64_t row = (int64_t)r * bits / 8;
#pragma omp parallel for schedule(static)
    for (int64_t v = 0; v < n_vec; ++v) {
        memset(packed + v * row, 0, (size_t)row);
        for (int j = 0; j < r; ++j) {
            int64_t y = 0;
            for (int t = 0; t < d; ++t)
                y += (int64_t)R[(int64_t)t * r + j] * quant8(load_f32(x, dtype, v * d + t), qscale);
            const int c = clampi(floor_div(y + ((int64_t)1 << (shift - 1)), (int64_t)1 << shift), -lim, lim);
            packed[v * row + j / per] |= (uint8_t)(((unsigned)c & ((1u << bits) - 1u)) << (bits * (j % per)));
        }
    }
    return 0;
}

/* packed [n_vec, r*bits/8] -> code [n_vec, r] int8: the entries of oracle_encode_packed, sign-extended. */
int oracle_unpack_codes(const uint8_t *packed, int64_t n_vec, int r, int bits, int8_t *code) {
    if (!packed || !code || r <= 0 || (bits != 2 && bits != 4 && bits != 8) || (r * bits) % 8 != 0) return -1;
    const int per = 8 / bits;
    const int64_t row = (int64_t)r * bits / 8;
    for (int64_t v = 0; v < n_vec; ++v)
        for (int j = 0; j < r; ++j) {
            int c = (packed[v * row + j / per] >> (bits * (j % per))) & ((1 << bits) - 1);
            if (c >= 1 << (bits - 1)) c -= 1 << bits;
            code[v * r + j] = (int8_t)c;
        }
    return 0;
}

static int64_t dot_i8(const int8_t *a, const int8_t *b, int r) {
    int64_t s = 0;
    for (int j = 0; j < r; ++j) s += (int64_t)a[j] * (int64_t)b[j];
    return s;
}

/* ------------------------------------------------------------------ TempCache */

/*
 * One frame of new tokens is merged into the per-head caches, every decision taken against the
 * cache as it was at entry.
 *
 * cache:   K, V [H,C,d] dtype; code [H,C,r]; cnt, stamp [H,C]; len [H]   (updated in place)
 * new:     K_new, V_new [H,n_new,d]; P_new (probe, NULL => K_new) [H,n_new,d]
 * cand:    [H,n_cand] slot ids that form the candidate SET of the match (ids outside [0,len) are ignored, the
 *          order of the list and repeated ids mean nothing), NULL => all live slots.  Of equally scored
 *          candidates the smallest slot wins (Sec. 5.2 names no order among ties; every tie here goes to the
 *          lowest index).
 * metric:  0 => S = 2 cp.code_j - |code_j|^2 (nearest in code space), 1 => S = cp.code_j
 * tau2_q16 = rint(tau^2 * 65536); merge iff dot > 0 and dot^2 * 65536 >= tau2_q16 * |a|^2 |b|^2 on the
 *          8-bit quantised full-width keys a (new) and b (cached)
 * rep_mode: representative key of a merged group (appendix, "Representative selection in KV merging"):
 *          0 => last key (the method's choice: the most recent member, here the group's winner of this frame),
 *          1 => mean key: the multiplicity-weighted mean of the group's keys.  The stored mean feeds later integer
 *               decisions (codes, the cosine test), so its arithmetic is fixed: float32, cnt * K_old first, then the
 *               members' keys added in ascending token order, one float32 division, one rounding to the storage
 *               type; the slot's code is the code of that stored key.
 *          2 => medoid key: of the group's members the one with the smallest total distance to the others.  A bounded
 *               cache keeps no members, so the group seen by one call is the slot's current representative, standing
 *               for the cnt tokens merged so far, and this frame's joiners (weight 1 each); distance = squared
 *               Euclidean distance of the 8-bit codes (an exact integer); cost(x) = sum over members y of
 *               weight(y) * dist(x, y); smallest cost wins, ties go to the current representative, then to the smaller
 *               token.  The current representative winning leaves key and code as they are (value, multiplicity and
 *               stamp are updated as always).
 * out:     merge_map [H,n_new] destination slot or -1 (dropped); merged [H,n_new] 0/1;
 *          stats [H,8] = len', n_merged, n_appended, n_evicted, n_dropped, 0, 0, 0
 */
int oracle_tempcache_compress(void *K, void *V, int8_t *code, int32_t *cnt, int32_t *stamp, int32_t *len, int H,
                              int C, int d, int r, int dtype, const int8_t *R, float qscale, int shift,
                              const void *K_new, const void *V_new, const void *P_new, int n_new,
                              const int32_t *cand, int n_cand, int metric, int32_t tau2_q16, int32_t frame_id,
                              int rep_mode, int32_t *merge_map, uint8_t *merged, int32_t *stats) {
    if (!K || !V || !code || !cnt || !stamp || !len || !R || !K_new || !V_new || !merge_map || !merged || !stats)
        return -1;
    if (H <= 0 || C <= 0 || d <= 0 || r <= 0 || n_new < 0 || (metric != 0 && metric != 1)) return -1;
    if (rep_mode != 0 && rep_mode != 1 && rep_mode != 2) return -1;
    if (!P_new) P_new = K_new;
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int h = 0; h < H; ++h) {
        const int L = len[h];
        const int64_t cb = (int64_t)h * C;     /* first slot of this head   */
        const int64_t nb = (int64_t)h * n_new; /* first new token of this head */
        int8_t *cp = malloc((size_t)(n_new > 0 ? n_new : 1) * r);
        int8_t *ck = malloc((size_t)(n_new > 0 ? n_new : 1) * r);
        uint8_t *is_cand = calloc((size_t)(L > 0 ? L : 1), 1);
        int32_t *jstar = malloc(sizeof(int32_t) * (size_t)(n_new > 0 ? n_new : 1));
        int64_t *sstar = malloc(sizeof(int64_t) * (size_t)(n_new > 0 ? n_new : 1));
        int32_t *group = calloc((size_t)(L > 0 ? L : 1), sizeof(int32_t));  /* |M_j| */
        int32_t *winner = malloc(sizeof(int32_t) * (size_t)(L > 0 ? L : 1));
        uint8_t *victim = calloc((size_t)(L > 0 ? L : 1), 1);
        if (!cp || !ck || !is_cand || !jstar || !sstar || !group || !winner || !victim) {
#pragma omp atomic write
            err = -5;
            goto done;
        }
        /* step 1: codes of the probes and of the new keys */
        for (int i = 0; i < n_new; ++i) {
            encode_vec(P_new, dtype, (nb + i) * d, d, R, r, qscale, shift, cp + (int64_t)i * r);
            encode_vec(K_new, dtype, (nb + i) * d, d, R, r, qscale, shift, ck + (int64_t)i * r);
        }
        /* step 2: candidate set, then the top-1 match over it in ascending slot order: the strict '>' keeps the
         * smallest slot among equally scored candidates */
        if (cand) {
            for (int c = 0; c < n_cand; ++c) {
                const int32_t j = cand[(int64_t)h * n_cand + c];
                if (j >= 0 && j < L) is_cand[j] = 1;
            }
        } else {
            for (int j = 0; j < L; ++j) is_cand[j] = 1;
        }
        for (int i = 0; i < n_new; ++i) {
            jstar[i] = -1;
            sstar[i] = 0;
            for (int j = 0; j < L; ++j) {
                if (!is_cand[j]) continue;
                const int8_t *cj = code + (cb + j) * r;
                int64_t S = dot_i8(cp + (int64_t)i * r, cj, r);
                if (metric == 0) S = 2 * S - dot_i8(cj, cj, r);
                if (jstar[i] < 0 || S > sstar[i]) {
                    jstar[i] = j;
                    sstar[i] = S;
                }
            }
        }
        /* step 3: cosine test on the 8-bit quantised full-width keys, as an integer inequality */
        int n_merged = 0;
        for (int i = 0; i < n_new; ++i) {
            merged[nb + i] = 0;
            if (jstar[i] < 0) continue;
            int64_t dot = 0, na = 0, nbb = 0;
            for (int t = 0; t < d; ++t) {
                int64_t a = quant8(load_f32(K_new, dtype, (nb + i) * d + t), qscale);
                int64_t b = quant8(load_f32(K, dtype, (cb + jstar[i]) * d + t), qscale);
                dot += a * b;
                na += a * a;
                nbb += b * b;
            }
            if (dot > 0 && dot * dot * 65536 >= (int64_t)tau2_q16 * na * nbb) {
                merged[nb + i] = 1;
                n_merged += 1;
            }
        }
        /* step 4: members of every touched slot and its winner: the joiner closest to the slot in code
         * space (metric 0: -|cp_i - code_j|^2 = S - |cp_i|^2; metric 1: S), then the smallest token index */
        for (int i = 0; i < n_new; ++i) {
            if (!merged[nb + i]) continue;
            if (metric == 0) sstar[i] -= dot_i8(cp + (int64_t)i * r, cp + (int64_t)i * r, r);
        }
        for (int i = 0; i < n_new; ++i) {
            if (!merged[nb + i]) continue;
            int j = jstar[i];
            if (group[j] == 0 || sstar[i] > sstar[winner[j]]) winner[j] = i;
            group[j] += 1;
        }
        /* step 5: tokens to append, evictions needed, victims = oldest untouched live slots */
        int n_unmerged = n_new - n_merged;
        int e = L + n_unmerged - C;
        if (e < 0) e = 0;
        int n_victims = 0;
        for (int pick = 0; pick < e; ++pick) { /* repeatedly take the smallest (stamp, slot) not yet taken */
            int best = -1;
            for (int j = 0; j < L; ++j) {
                if (group[j] != 0 || victim[j]) continue;
                if (best < 0 || stamp[cb + j] < stamp[cb + best]) best = j;
            }
            if (best < 0) break;
            victim[best] = 1;
            n_victims += 1;
        }
        int n_dropped = e - n_victims;
        /* step 6a: merged groups: mean value with multiplicity, most recent key as representative */
        {
            /* value sums: cnt * V_old first, then the members' values in ascending token order */
            double *acc = malloc(sizeof(double) * (size_t)(n_merged > 0 ? n_merged : 1) * d);
            int32_t *row_of = malloc(sizeof(int32_t) * (size_t)(L > 0 ? L : 1)); /* slot -> row of acc */
            int n_rows = 0;
            for (int j = 0; j < L; ++j) row_of[j] = -1;
            for (int i = 0; i < n_new; ++i) {
                if (!merged[nb + i]) continue;
                int j = jstar[i];
                merge_map[nb + i] = j;
                if (row_of[j] < 0) {
                    row_of[j] = n_rows++;
                    for (int t = 0; t < d; ++t)
                        acc[(int64_t)row_of[j] * d + t] =
                            (double)cnt[cb + j] * (double)load_f32(V, dtype, (cb + j) * d + t);
                }
                for (int t = 0; t < d; ++t)
                    acc[(int64_t)row_of[j] * d + t] += (double)load_f32(V_new, dtype, (nb + i) * d + t);
            }
            for (int j = 0; j < L; ++j) {
                if (group[j] == 0) continue;
                for (int t = 0; t < d; ++t)
                    store_val(V, dtype, (cb + j) * d + t,
                              acc[(int64_t)row_of[j] * d + t] / (double)(cnt[cb + j] + group[j]));
                if (rep_mode == 0) {
                    copy_row(K, cb + j, K_new, nb + winner[j], d, dtype);
                    memcpy(code + (cb + j) * r, ck + (int64_t)winner[j] * r, (size_t)r);
                } else if (rep_mode == 2) {
                    /* medoid over {current representative (weight cnt)} and the joiners (weight 1), candidates in the
                     * order representative, then tokens ascending; strict '<' keeps the earlier candidate on ties */
                    const int8_t *cold = code + (cb + j) * r;
                    int best = -1; /* -1 = the current representative */
                    int64_t best_cost = 0;
                    for (int i = 0; i < n_new; ++i)
                        if (merged[nb + i] && jstar[i] == j) {
                            const int8_t *ci = ck + (int64_t)i * r;
                            best_cost += dot_i8(cold, cold, r) + dot_i8(ci, ci, r) - 2 * dot_i8(cold, ci, r);
                        }
                    for (int a = 0; a < n_new; ++a) {
                        if (!(merged[nb + a] && jstar[a] == j)) continue;
                        const int8_t *ca = ck + (int64_t)a * r;
                        int64_t cost = (int64_t)cnt[cb + j] * (dot_i8(ca, ca, r) + dot_i8(cold, cold, r) - 2 * dot_i8(ca, cold, r));
                        for (int i = 0; i < n_new; ++i)
                            if (merged[nb + i] && jstar[i] == j) {
                                const int8_t *ci = ck + (int64_t)i * r;
                                cost += dot_i8(ca, ca, r) + dot_i8(ci, ci, r) - 2 * dot_i8(ca, ci, r);
                            }
                        if (cost < best_cost) {
                            best = a;
                            best_cost = cost;
                        }
                    }
                    if (best >= 0) {
                        copy_row(K, cb + j, K_new, nb + best, d, dtype);
                        memcpy(code + (cb + j) * r, ck + (int64_t)best * r, (size_t)r);
                    }
                } else {
                    for (int t = 0; t < d; ++t) {
                        volatile float ksum = (float)cnt[cb + j] * load_f32(K, dtype, (cb + j) * d + t);
                        for (int i = 0; i < n_new; ++i)
                            if (merged[nb + i] && jstar[i] == j) ksum = ksum + load_f32(K_new, dtype, (nb + i) * d + t);
                        volatile float kmean = ksum / (float)(cnt[cb + j] + group[j]);
                        if (dtype == 0)
                            ((float *)K)[(cb + j) * d + t] = kmean;
                        else
                            ((uint16_t *)K)[(cb + j) * d + t] = f32_to_bf16(kmean);
                    }
                    encode_vec(K, dtype, (cb + j) * d, d, R, r, qscale, shift, code + (cb + j) * r);
                }
                cnt[cb + j] += group[j];
                stamp[cb + j] = frame_id;
            }
            free(acc);
            free(row_of);
        }
        /* step 6b: unmerged tokens in ascending order: first into the victims (ascending slot), then
         * into fresh slots; the last n_dropped of them do not fit and are dropped */
        int a = 0, next_victim = 0;
        for (int i = 0; i < n_new; ++i) {
            if (merged[nb + i]) continue;
            int dst;
            if (a >= n_unmerged - n_dropped) {
                dst = -1;
            } else if (a < n_victims) {
                while (!victim[next_victim]) next_victim += 1;
                dst = next_victim;
                next_victim += 1;
            } else {
                dst = L + (a - n_victims);
            }
            merge_map[nb + i] = dst;
            if (dst >= 0) {
                copy_row(K, cb + dst, K_new, nb + i, d, dtype);
                copy_row(V, cb + dst, V_new, nb + i, d, dtype);
                memcpy(code + (cb + dst) * r, ck + (int64_t)i * r, (size_t)r);
                cnt[cb + dst] = 1;
                stamp[cb + dst] = frame_id;
            }
            a += 1;
        }
        {
            int n_app = n_unmerged - n_dropped;
            int newL = L + n_app - n_victims;
            len[h] = newL;
            int32_t *st = stats + (int64_t)h * 8;
            st[0] = newL;
            st[1] = n_merged;
            st[2] = n_app;
            st[3] = n_victims;
            st[4] = n_dropped;
            st[5] = st[6] = st[7] = 0;
        }
    done:
        free(cp);
        free(ck);
        free(is_cand);
        free(jstar);
        free(sstar);
        free(group);
        free(winner);
        free(victim);
    }
    return err;
}

/* ------------------------------------------------------------------ ANN selection */

/* Pick the n_out largest scores (ties: smaller index), flag them; O(n_out * n) on purpose. */
static void pick_top(const int64_t *score, int n, int n_out, uint8_t *picked) {
    memset(picked, 0, (size_t)(n > 0 ? n : 1));
    for (int t = 0; t < n_out; ++t) {
        int best = -1;
        for (int k = 0; k < n; ++k) {
            if (picked[k]) continue;
            if (best < 0 || score[k] > score[best]) best = k;
        }
        if (best < 0) break;
        picked[best] = 1;
    }
}

/*
 * AnnSA.  qcode [H,n_q,r], kcode [H,C,r], len [H].
 * Query block b (BQ queries) is summarised by n_rep mean codes, one per run of g = BQ/n_rep
 * queries: rep = floor((sum of codes + floor(g/2)) / g)  (runs with no query are skipped).
 * Score of key block kb (BK keys) = max over summaries and over its live keys of rep . code_k.
 * The min(n_sel, ceil(len/BK)) best key blocks are written in ascending order to
 * sel [H,n_qb,n_sel] (-1 padded), their number to nsel [H,n_qb].
 */
/*
 * The same with forced blocks (Sec. 2: rolling-window generators keep the first frames as an attention sink; a local
 * window is the usual companion): the first n_sink key blocks and the last n_local live key blocks of every head are
 * always among the selected ones and count against the budget (n_sink + n_local <= n_sel); the rest of the budget goes
 * to the best-scoring other blocks as before.  n_sink = n_local = 0 is oracle_ann_select_self.
 */
int oracle_ann_select_self_forced(const int8_t *qcode, int n_q, const int8_t *kcode, const int32_t *len, int H, int C,
                                  int r, int BQ, int n_rep, int BK, int n_sel, int n_sink, int n_local, int32_t *sel,
                                  int32_t *nsel) {
    if (!qcode || !kcode || !len || !sel || !nsel) return -1;
    if (H <= 0 || C <= 0 || r <= 0 || BQ <= 0 || n_rep <= 0 || BK <= 0 || n_sel <= 0 || BQ % n_rep != 0) return -1;
    if (n_sink < 0 || n_local < 0 || n_sink + n_local > n_sel) return -1;
    const int n_qb = (n_q + BQ - 1) / BQ;
    const int g = BQ / n_rep;
    const int n_kb_cap = (C + BK - 1) / BK;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int h = 0; h < H; ++h) {
        for (int b = 0; b < n_qb; ++b) {
            const int L = len[h];
            const int n_kb = (L + BK - 1) / BK;
            int64_t *rep = malloc(sizeof(int64_t) * (size_t)n_rep * r);
            uint8_t *rep_ok = malloc((size_t)n_rep);
            int64_t *score = malloc(sizeof(int64_t) * (size_t)(n_kb_cap > 0 ? n_kb_cap : 1));
            uint8_t *picked = malloc((size_t)(n_kb_cap > 0 ? n_kb_cap : 1));
            for (int u = 0; u < n_rep; ++u) {
                int q0 = b * BQ + u * g, q1 = q0 + g;
                if (q1 > n_q) q1 = n_q;
                rep_ok[u] = q0 < n_q;
                for (int j = 0; j < r; ++j) {
                    int64_t s = 0;
                    for (int q = q0; q < q1; ++q) s += qcode[((int64_t)h * n_q + q) * r + j];
                    rep[(int64_t)u * r + j] = floor_div(s + g / 2, g);
                }
            }
            for (int kb = 0; kb < n_kb; ++kb) {
                int have = 0;
                int64_t best = 0;
                for (int k = kb * BK; k < (kb + 1) * BK && k < L; ++k) {
                    const int8_t *ck = kcode + ((int64_t)h * C + k) * r;
                    for (int u = 0; u < n_rep; ++u) {
                        if (!rep_ok[u]) continue;
                        int64_t s = 0;
                        for (int j = 0; j < r; ++j) s += rep[(int64_t)u * r + j] * (int64_t)ck[j];
                        if (!have || s > best) {
                            best = s;
                            have = 1;
                        }
                    }
                }
                score[kb] = best;
                if (kb < n_sink || kb >= n_kb - n_local) score[kb] = INT64_MAX; /* forced: ahead of every real score */
            }
            int n_out = n_sel < n_kb ? n_sel : n_kb;
            pick_top(score, n_kb, n_out, picked);
            int32_t *out = sel + ((int64_t)h * n_qb + b) * n_sel;
            int w = 0;
            for (int kb = 0; kb < n_kb; ++kb)
                if (picked[kb]) out[w++] = kb;
            nsel[(int64_t)h * n_qb + b] = w;
            for (; w < n_sel; ++w) out[w] = -1;
            free(rep);
            free(rep_ok);
            free(score);
            free(picked);
        }
    }
    return 0;
}

int oracle_ann_select_self(const int8_t *qcode, int n_q, const int8_t *kcode, const int32_t *len, int H, int C, int r,
                           int BQ, int n_rep, int BK, int n_sel, int32_t *sel, int32_t *nsel) {
    return oracle_ann_select_self_forced(qcode, n_q, kcode, len, H, C, r, BQ, n_rep, BK, n_sel, 0, 0, sel, nsel);
}

/*
 * AnnCA.  qcode [H,n_q,r], pcode [H,n_p,r].
 * Score of prompt token p for query block b = max over the block's queries of c_q . c_p (a token
 * is kept when at least one query of the block is its neighbour).  The min(n_sel, n_p) best
 * tokens go to sel [H,n_qb,n_sel] in ascending order (-1 padded), their number to nsel.
 */
int oracle_ann_select_cross(const int8_t *qcode, int n_q, const int8_t *pcode, int n_p, int H, int r, int BQ,
                            int n_sel, int32_t *sel, int32_t *nsel) {
    if (!qcode || !pcode || !sel || !nsel) return -1;
    if (H <= 0 || n_p < 0 || r <= 0 || BQ <= 0 || n_sel <= 0) return -1;
    const int n_qb = (n_q + BQ - 1) / BQ;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int h = 0; h < H; ++h) {
        for (int b = 0; b < n_qb; ++b) {
            int64_t *score = malloc(sizeof(int64_t) * (size_t)(n_p > 0 ? n_p : 1));
            uint8_t *picked = malloc((size_t)(n_p > 0 ? n_p : 1));
            int q0 = b * BQ, q1 = q0 + BQ;
            if (q1 > n_q) q1 = n_q;
            for (int p = 0; p < n_p; ++p) {
                const int8_t *cpp = pcode + ((int64_t)h * n_p + p) * r;
                int64_t best = 0;
                for (int q = q0; q < q1; ++q) {
                    int64_t s = dot_i8(qcode + ((int64_t)h * n_q + q) * r, cpp, r);
                    if (q == q0 || s > best) best = s;
                }
                score[p] = best;
            }
            int n_out = n_sel < n_p ? n_sel : n_p;
            pick_top(score, n_p, n_out, picked);
            int32_t *out = sel + ((int64_t)h * n_qb + b) * n_sel;
            int w = 0;
            for (int p = 0; p < n_p; ++p)
                if (picked[p]) out[w++] = p;
            nsel[(int64_t)h * n_qb + b] = w;
            for (; w < n_sel; ++w) out[w] = -1;
            free(score);
            free(picked);
        }
    }
    return 0;
}

/* ------------------------------------------------------------------ prompt-induced buckets (AnnCA -> AnnSA) */
/*
 * Sec. 5.4: self-attention reuses the semantic buckets found during cross-attention pruning (Sec. 5.3); a query is
 * assigned to one or more buckets and attends only to keys of the same bucket(s).  Reading: the prompt tokens are the
 * buckets.  A code belongs to the m prompt tokens with the largest code inner product c . c_p (the same products
 * AnnCA ranks prompt tokens by), ties to the smaller token id.
 * code [H,n,r], pcode [H,n_p,r] -> bucket [H,n,m] (token ids, best first; -1 where n_p < m).
 */
int oracle_prompt_buckets(const int8_t *code, int n, const int8_t *pcode, int n_p, int H, int r, int m,
                          int32_t *bucket) {
    if (!code || !pcode || !bucket) return -1;
    if (H <= 0 || n < 0 || n_p < 0 || r <= 0 || m <= 0) return -1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int h = 0; h < H; ++h) {
        int64_t *score = malloc(sizeof(int64_t) * (size_t)(n_p > 0 ? n_p : 1));
        uint8_t *taken = malloc((size_t)(n_p > 0 ? n_p : 1));
        for (int i = 0; i < n; ++i) {
            const int8_t *c = code + ((int64_t)h * n + i) * r;
            for (int p = 0; p < n_p; ++p) score[p] = dot_i8(c, pcode + ((int64_t)h * n_p + p) * r, r);
            memset(taken, 0, (size_t)(n_p > 0 ? n_p : 1));
            for (int j = 0; j < m; ++j) {
                int best = -1;
                for (int p = 0; p < n_p; ++p) {
                    if (taken[p]) continue;
                    if (best < 0 || score[p] > score[best]) best = p;
                }
                if (best >= 0) taken[best] = 1;
                bucket[((int64_t)h * n + i) * m + j] = best;
            }
        }
        free(score);
        free(taken);
    }
    return 0;
}

/*
 * AnnSA on those buckets.  qbucket [H,n_q,m], kbucket [H,C,m] (entries -1 are ignored), len [H].
 * A query block owns the buckets of its queries, a key block those of its live keys; the score of a key block is the
 * number of buckets the two share.  Only key blocks that share at least one bucket are candidates ("only keys within
 * the same bucket(s)"); of these the n_sel with the largest score are kept (ties: smaller block), written ascending
 * to sel [H,n_qb,n_sel] (-1 padded), their number to nsel.  The first n_sink and the last n_local live key blocks
 * are always kept and count against the budget, as in oracle_ann_select_self_forced.
 */
int oracle_ann_select_buckets(const int32_t *qbucket, int n_q, const int32_t *kbucket, const int32_t *len, int H,
                              int C, int m, int n_p, int BQ, int BK, int n_sel, int n_sink, int n_local,
                              int32_t *sel, int32_t *nsel) {
    if (!qbucket || !kbucket || !len || !sel || !nsel) return -1;
    if (H <= 0 || C <= 0 || m <= 0 || n_p <= 0 || BQ <= 0 || BK <= 0 || n_sel <= 0) return -1;
    if (n_sink < 0 || n_local < 0 || n_sink + n_local > n_sel) return -1;
    const int n_qb = (n_q + BQ - 1) / BQ;
    const int n_kb_cap = (C + BK - 1) / BK;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int h = 0; h < H; ++h) {
        for (int b = 0; b < n_qb; ++b) {
            const int L = len[h] < C ? len[h] : C;
            const int n_kb = (L + BK - 1) / BK;
            uint8_t *own = calloc((size_t)n_p, 1);
            uint8_t *has = malloc((size_t)n_p);
            int64_t *score = malloc(sizeof(int64_t) * (size_t)(n_kb_cap > 0 ? n_kb_cap : 1));
            uint8_t *picked = malloc((size_t)(n_kb_cap > 0 ? n_kb_cap : 1));
            for (int q = b * BQ; q < (b + 1) * BQ && q < n_q; ++q)
                for (int j = 0; j < m; ++j) {
                    const int32_t t = qbucket[((int64_t)h * n_q + q) * m + j];
                    if (t >= 0 && t < n_p) own[t] = 1;
                }
            int n_cand = 0;
            for (int kb = 0; kb < n_kb; ++kb) {
                memset(has, 0, (size_t)n_p);
                for (int k = kb * BK; k < (kb + 1) * BK && k < L; ++k)
                    for (int j = 0; j < m; ++j) {
                        const int32_t t = kbucket[((int64_t)h * C + k) * m + j];
                        if (t >= 0 && t < n_p) has[t] = 1;
                    }
                int64_t shared = 0;
                for (int t = 0; t < n_p; ++t) shared += own[t] && has[t];
                const int forced = kb < n_sink || kb >= n_kb - n_local;
                score[kb] = forced ? INT64_MAX : (shared > 0 ? shared : -1); /* -1: shares nothing, no candidate */
                n_cand += forced || shared > 0;
            }
            const int n_out = n_sel < n_cand ? n_sel : n_cand;
            pick_top(score, n_kb, n_out, picked);
            int32_t *out = sel + ((int64_t)h * n_qb + b) * n_sel;
            int w = 0;
            for (int kb = 0; kb < n_kb; ++kb)
                if (picked[kb]) out[w++] = kb;
            nsel[(int64_t)h * n_qb + b] = w;
            for (; w < n_sel; ++w) out[w] = -1;
            free(own);
            free(has);
            free(score);
            free(picked);
        }
    }
    return 0;
}

/* ------------------------------------------------------------------ sign codes (LSH family) */

/*
 * x [n_vec, d] -> bits [n_vec, n_bits/32] (uint32 words, bit j of a vector in word j/32 at position j%32).
 * Bit j = 1 iff sum_t R[t][j] * xq[t] >= 0, with xq the 8-bit quantisation of oracle_encode and R [d, n_bits]
 * a +-1 matrix: the side of the j-th random hyperplane the (quantised) vector lies on.
 */
int oracle_encode_sign(const void *x, int dtype, int64_t n_vec, int d, const int8_t *R, int n_bits, float qscale,
                       uint32_t *bits) {
    if (!x || !R || !bits || d <= 0 || n_bits <= 0 || n_bits % 32 != 0) return -1;
    const int W = n_bits / 32;
#pragma omp parallel for schedule(static)
    for (int64_t v = 0; v < n_vec; ++v) {
        for (int w = 0; w < W; ++w) bits[v * W + w] = 0u;
        for (int j = 0; j < n_bits; ++j) {
            int64_t y = 0;
            for (int t = 0; t < d; ++t)
                y += (int64_t)R[(int64_t)t * n_bits + j] * quant8(load_f32(x, dtype, v * d + t), qscale);
            if (y >= 0) bits[v * W + j / 32] |= (uint32_t)1 << (j % 32);
        }
    }
    return 0;
}

static int equal_bits(const uint32_t *a, const uint32_t *b, int W) {
    int n = 0;
    for (int w = 0; w < W; ++w) {
        uint32_t x = ~(a[w] ^ b[w]);
        while (x) {
            n += (int)(x & 1u);
            x >>= 1;
        }
    }
    return n;
}

/*
 * Selection on sign codes.  qbits [H,n_q,W], kbits [H,C,W] (W = n_bits/32), len [H].
 * Query block b (BQ queries) is summarised by n_rep majority codes, one per run of g = BQ/n_rep queries: bit j of a
 * summary is 1 iff at least half of the run's queries have it set (2 * ones >= queries in the run; runs with no
 * query are skipped).  Score of key block kb (BK keys) = max over summaries and over its live keys of the number
 * of equal bits.  The min(n_sel, ceil(len/BK)) best key blocks (ties: lowest index) are written in ascending
 * order to sel [H,n_qb,n_sel] (-1 padded), their number to nsel [H,n_qb].
 * n_rep = BQ and BK = 1 give the cross-attention form: a key is scored by its best-matching query of the block.
 */
/* Tables in which two hash codes fall into the same bucket, or into buckets at most `radius` bits apart: the code is
 * cut into bands of band_bits consecutive bits, one band per table. */
static int colliding_tables(const uint32_t *a, const uint32_t *b, int n_bits, int band_bits, int radius) {
    int n = 0;
    for (int t = 0; t < n_bits / band_bits; ++t) {
        int diff = 0;
        for (int j = t * band_bits; j < (t + 1) * band_bits; ++j)
            diff += (int)(((a[j / 32] ^ b[j / 32]) >> (j % 32)) & 1u);
        n += diff <= radius;
    }
    return n;
}

/* band_bits = 0: pairs are scored by their equal bits and every key block is a candidate (oracle_ann_select_lsh);
 * band_bits > 0: pairs are scored by their colliding tables and only key blocks with a collision are candidates. */
static int lsh_select(const uint32_t *qbits, int n_q, const uint32_t *kbits, const int32_t *len, int H, int C,
                      int n_bits, int band_bits, int radius, int BQ, int n_rep, int BK, int n_sel, int n_sink,
                      int n_local, int32_t *sel, int32_t *nsel) {
    if (!qbits || !kbits || !len || !sel || !nsel) return -1;
    if (H <= 0 || C <= 0 || n_bits <= 0 || n_bits % 32 != 0 || BQ <= 0 || n_rep <= 0 || BK <= 0 || n_sel <= 0 ||
        BQ % n_rep != 0)
        return -1;
    if (band_bits < 0 || (band_bits > 0 && n_bits % band_bits != 0) || radius < 0) return -1;
    if (n_sink < 0 || n_local < 0 || n_sink + n_local > n_sel) return -1;
    const int W = n_bits / 32;
    const int n_qb = (n_q + BQ - 1) / BQ;
    const int g = BQ / n_rep;
    const int n_kb_cap = (C + BK - 1) / BK;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int h = 0; h < H; ++h) {
        for (int b = 0; b < n_qb; ++b) {
            const int L = len[h] < C ? len[h] : C;
            const int n_kb = (L + BK - 1) / BK;
            uint32_t *rep = calloc((size_t)n_rep * W, sizeof(uint32_t));
            uint8_t *rep_ok = malloc((size_t)n_rep);
            int64_t *score = malloc(sizeof(int64_t) * (size_t)(n_kb_cap > 0 ? n_kb_cap : 1));
            uint8_t *picked = malloc((size_t)(n_kb_cap > 0 ? n_kb_cap : 1));
            for (int u = 0; u < n_rep; ++u) {
                int q0 = b * BQ + u * g, q1 = q0 + g;
                if (q1 > n_q) q1 = n_q;
                rep_ok[u] = q0 < n_q;
                for (int j = 0; j < n_bits && rep_ok[u]; ++j) {
                    int ones = 0;
                    for (int q = q0; q < q1; ++q)
                        ones += (int)((qbits[((int64_t)h * n_q + q) * W + j / 32] >> (j % 32)) & 1u);
                    if (2 * ones >= q1 - q0) rep[(int64_t)u * W + j / 32] |= (uint32_t)1 << (j % 32);
                }
            }
            int n_cand = 0;
            for (int kb = 0; kb < n_kb; ++kb) {
                int64_t best = -1;
                for (int k = kb * BK; k < (kb + 1) * BK && k < L; ++k)
                    for (int u = 0; u < n_rep; ++u) {
                        if (!rep_ok[u]) continue;
                        const uint32_t *ck = kbits + ((int64_t)h * C + k) * W;
                        int64_t s = band_bits ? colliding_tables(rep + (int64_t)u * W, ck, n_bits, band_bits, radius)
                                              : equal_bits(rep + (int64_t)u * W, ck, W);
                        if (s > best) best = s;
                    }
                const int forced = kb < n_sink || kb >= n_kb - n_local;
                if (band_bits && best < 1) best = -1; /* no table in common: not a candidate */
                n_cand += forced || !band_bits || best >= 1;
                score[kb] = forced ? INT64_MAX : best;
            }
            int n_out = n_sel < n_cand ? n_sel : n_cand;
            pick_top(score, n_kb, n_out, picked);
            int32_t *out = sel + ((int64_t)h * n_qb + b) * n_sel;
            int w = 0;
            for (int kb = 0; kb < n_kb; ++kb)
                if (picked[kb]) out[w++] = kb;
            nsel[(int64_t)h * n_qb + b] = w;
            for (; w < n_sel; ++w) out[w] = -1;
            free(rep);
            free(rep_ok);
            free(score);
            free(picked);
        }
    }
    return 0;
}

int oracle_ann_select_lsh(const uint32_t *qbits, int n_q, const uint32_t *kbits, const int32_t *len, int H, int C,
                          int n_bits, int BQ, int n_rep, int BK, int n_sel, int32_t *sel, int32_t *nsel) {
    return lsh_select(qbits, n_q, kbits, len, H, C, n_bits, 0, 0, BQ, n_rep, BK, n_sel, 0, 0, sel, nsel);
}

/*
 * Bucket form of the same selection (Sec. 5.1, LSH paragraph: a query only compares against keys that land in the same
 * bucket(s); Sec. 2 names multi-table bucket probing).  The n_bits hash bits are cut into n_bits / band_bits bands,
 * one hash table each; a vector's bucket in a table is its band.  A summary and a key collide in a table when their
 * buckets are equal (radius 0) or differ in at most `radius` bits (multi-probe: the query side also looks into the
 * neighbouring buckets).  Score of a pair = number of tables in which it collides; score of a key block = best pair
 * over the block's summaries and its live keys; a key block without any collision is no candidate; of the candidates
 * the n_sel best are kept (ties: lowest index).  The first n_sink / last n_local live blocks are always kept.
 */
int oracle_ann_select_lsh_buckets(const uint32_t *qbits, int n_q, const uint32_t *kbits, const int32_t *len, int H,
                                  int C, int n_bits, int band_bits, int radius, int BQ, int n_rep, int BK, int n_sel,
                                  int n_sink, int n_local, int32_t *sel, int32_t *nsel) {
    if (band_bits <= 0) return -1;
    return lsh_select(qbits, n_q, kbits, len, H, C, n_bits, band_bits, radius, BQ, n_rep, BK, n_sel, n_sink, n_local,
                      sel, nsel);
}

/* ------------------------------------------------------------------ sparse attention */

/* Collect the live key indices of the key blocks listed for query block b. Returns their number. */
static int gather_keys(const int32_t *sel_row, int n_listed, int BK, int L, int32_t *keys) {
    int n = 0;
    const int n_kb = (L + BK - 1) / BK;
    for (int s = 0; s < n_listed; ++s) {
        int kb = sel_row[s];
        if (kb < 0 || kb >= n_kb) continue;
        for (int k = kb * BK; k < (kb + 1) * BK && k < L; ++k) keys[n++] = k;
    }
    return n;
}

/*
 * Q [H,n_q,d], K,V [H,C,d] (dtype), cnt [H,C] or NULL, len [H], sel [H,n_qb,n_sel], nsel [H,n_qb].
 * For query i of block b over the live keys J of the listed key blocks:
 *   l_j = scale * (q_i . k_j) + ln(cnt_j),  o_i = sum_j softmax(l)_j v_j,  lse_i = ln sum_j exp(l_j).
 * O [H,n_q,d] and lse [H,n_q] are returned in fp64.  J empty => o = 0, lse = -inf.
 */
int oracle_sparse_attn_fwd(const void *Q, int n_q, const void *K, const void *V, const int32_t *cnt,
                           const int32_t *len, int H, int C, int d, int dtype, const int32_t *sel,
                           const int32_t *nsel, int BQ, int BK, int n_sel, double scale, double *O, double *lse) {
    if (!Q || !K || !V || !len || !sel || !nsel || !O) return -1;
    if (H <= 0 || C <= 0 || d <= 0 || BQ <= 0 || BK <= 0 || n_sel <= 0) return -1;
    const int n_qb = (n_q + BQ - 1) / BQ;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int h = 0; h < H; ++h) {
        for (int b = 0; b < n_qb; ++b) {
            const int L = len[h];
            const int32_t *row = sel + ((int64_t)h * n_qb + b) * n_sel;
            int n_listed = nsel[(int64_t)h * n_qb + b];
            if (n_listed > n_sel) n_listed = n_sel;
            int32_t *keys = malloc(sizeof(int32_t) * ((size_t)n_sel * BK + 1));
            double *logit = malloc(sizeof(double) * ((size_t)n_sel * BK + 1));
            const int nk = gather_keys(row, n_listed, BK, L, keys);
            for (int i = b * BQ; i < (b + 1) * BQ && i < n_q; ++i) {
                const int64_t qb = ((int64_t)h * n_q + i) * d;
                double mx = -INFINITY;
                for (int a = 0; a < nk; ++a) {
                    const int64_t kb = ((int64_t)h * C + keys[a]) * d;
                    double s = 0.0;
                    for (int t = 0; t < d; ++t) s += (double)load_f32(Q, dtype, qb + t) * (double)load_f32(K, dtype, kb + t);
                    s *= scale;
                    if (cnt) s += log((double)cnt[(int64_t)h * C + keys[a]]);
                    logit[a] = s;
                    if (s > mx) mx = s;
                }
                double den = 0.0;
                for (int a = 0; a < nk; ++a) {
                    logit[a] = exp(logit[a] - mx);
                    den += logit[a];
                }
                for (int t = 0; t < d; ++t) {
                    double acc = 0.0;
                    for (int a = 0; a < nk; ++a)
                        acc += logit[a] * (double)load_f32(V, dtype, ((int64_t)h * C + keys[a]) * d + t);
                    O[qb + t] = nk > 0 ? acc / den : 0.0;
                }
                if (lse) lse[(int64_t)h * n_q + i] = nk > 0 ? mx + log(den) : -INFINITY;
            }
            free(keys);
            free(logit);
        }
    }
    return 0;
}

/*
 * Attention recall and density of a selection, on every q_stride-th query:
 *   recall  = mean over queries of (softmax mass of the dense attention over all live keys that
 *             falls on the selected keys);
 *   density = selected query-key pairs / all query-key pairs.
 * Logits carry the ln(cnt) shift when cnt is given.  out[0] = recall, out[1] = density.
 */
int oracle_recall_density(const void *Q, int n_q, const void *K, const int32_t *cnt, const int32_t *len, int H, int C,
                          int d, int dtype, const int32_t *sel, const int32_t *nsel, int BQ, int BK, int n_sel,
                          double scale, int q_stride, double *out) {
    if (!Q || !K || !len || !sel || !nsel || !out || q_stride <= 0) return -1;
    const int n_qb = (n_q + BQ - 1) / BQ;
    double recall_sum = 0.0, pairs_sel = 0.0, pairs_all = 0.0;
    int64_t n_queries = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 4) reduction(+ : recall_sum, pairs_sel, pairs_all, n_queries)
    for (int h = 0; h < H; ++h) {
        for (int i = 0; i < n_q; ++i) {
            if (i % q_stride != 0) continue;
            const int L = len[h];
            if (L <= 0) continue;
            const int b = i / BQ;
            const int32_t *row = sel + ((int64_t)h * n_qb + b) * n_sel;
            int n_listed = nsel[(int64_t)h * n_qb + b];
            uint8_t *in_sel = calloc((size_t)L, 1);
            double *logit = malloc(sizeof(double) * (size_t)L);
            const int n_kb = (L + BK - 1) / BK;
            for (int s = 0; s < n_listed && s < n_sel; ++s) {
                int kb = row[s];
                if (kb < 0 || kb >= n_kb) continue;
                for (int k = kb * BK; k < (kb + 1) * BK && k < L; ++k) in_sel[k] = 1;
            }
            const int64_t qb = ((int64_t)h * n_q + i) * d;
            double mx = -INFINITY;
            for (int k = 0; k < L; ++k) {
                double s = 0.0;
                for (int t = 0; t < d; ++t)
                    s += (double)load_f32(Q, dtype, qb + t) * (double)load_f32(K, dtype, ((int64_t)h * C + k) * d + t);
                s *= scale;
                if (cnt) s += log((double)cnt[(int64_t)h * C + k]);
                logit[k] = s;
                if (s > mx) mx = s;
            }
            double den = 0.0, kept = 0.0, nsel_keys = 0.0;
            for (int k = 0; k < L; ++k) {
                double e = exp(logit[k] - mx);
                den += e;
                if (in_sel[k]) {
                    kept += e;
                    nsel_keys += 1.0;
                }
            }
            recall_sum += kept / den;
            pairs_sel += nsel_keys;
            pairs_all += (double)L;
            n_queries += 1;
            free(in_sel);
            free(logit);
        }
    }
    out[0] = n_queries ? recall_sum / (double)n_queries : 0.0;
    out[1] = pairs_all > 0 ? pairs_sel / pairs_all : 0.0;
    return 0;
}

/* ------------------------------------------------------------------ 8-bit floating-point K/V (E4M3) */

/* Value of an E4M3 code (OCP FN variant): sign bit, 4 exponent bits with bias 7, 3 mantissa bits; exponent 0 holds
 * the subnormals m/8 * 2^-6; the all-ones pattern of exponent and mantissa is NaN; there is no infinity. */
static double fp8_value(uint8_t c) {
    const int sign = c >> 7, e = (c >> 3) & 15, m = c & 7;
    double v;
    if (e == 15 && m == 7) return NAN;
    if (e == 0)
        v = ldexp((double)m / 8.0, -6);
    else
        v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return sign ? -v : v;
}

/* Nearest E4M3 code of a finite x, ties to the even mantissa, magnitudes beyond the largest finite value (448)
 * saturate to it.  Found by plain search over the 127 non-negative finite codes, not by bit tricks. */
static uint8_t fp8_code(float x) {
    const double a = fabs((double)x);
    int best = 0;
    double best_err = a; /* code 0 = +0 */
    for (int c = 1; c <= 0x7E; ++c) {
        const double err = fabs(a - fp8_value((uint8_t)c));
        if (err < best_err || (err == best_err && (c & 1) == 0 && (best & 1) == 1)) {
            best = c;
            best_err = err;
        }
    }
    if (a >= 448.0) best = 0x7E;
    return (uint8_t)(best | (signbit(x) ? 0x80 : 0));
}

int oracle_fp8_encode(const float *x, int64_t n, uint8_t *code) {
    if (!x || !code) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) code[i] = fp8_code(x[i]);
    return 0;
}

int oracle_fp8_decode(const uint8_t *code, int64_t n, double *x) {
    if (!x || !code) return -1;
    for (int64_t i = 0; i < n; ++i) x[i] = fp8_value(code[i]);
    return 0;
}

/*
 * The 8-bit copy of the cache that the fp8 attention reads, in its layout:
 *   K8  [H, Cp, d]            E4M3 code of every key coordinate, rows as in K (Cp = C rounded up to a multiple of 64)
 *   V8T [H, Cp/64, d, 64]     per block of 64 slots the values transposed: element (h, blk, t, j) = V[h][64 blk + j][t]
 * Only the blocks that hold a live slot whose stamp is >= stamp_lo are (re)written, whole: their live slots with the
 * codes of the stored K / V, their dead slots (>= len) with zero.  stamp_lo <= the smallest stamp rewrites everything.
 */
int oracle_kv_to_fp8(const void *K, const void *V, const int32_t *stamp, const int32_t *len, int H, int C, int d,
                     int dtype, int32_t stamp_lo, uint8_t *K8, uint8_t *V8T) {
    if (!K || !V || !stamp || !len || !K8 || !V8T || H <= 0 || C <= 0 || d <= 0) return -1;
    const int n_blk = (C + 63) / 64;
    const int64_t Cp = (int64_t)n_blk * 64;
#pragma omp parallel for collapse(2) schedule(static)
    for (int h = 0; h < H; ++h) {
        for (int blk = 0; blk < n_blk; ++blk) {
            const int L = len[h] < C ? len[h] : C;
            int dirty = 0;
            for (int j = 0; j < 64; ++j) {
                const int slot = blk * 64 + j;
                if (slot < L && stamp[(int64_t)h * C + slot] >= stamp_lo) dirty = 1;
            }
            if (!dirty) continue;
            for (int j = 0; j < 64; ++j) {
                const int slot = blk * 64 + j;
                for (int t = 0; t < d; ++t) {
                    uint8_t ck = 0, cv = 0;
                    if (slot < L) {
                        ck = fp8_code(load_f32(K, dtype, ((int64_t)h * C + slot) * d + t));
                        cv = fp8_code(load_f32(V, dtype, ((int64_t)h * C + slot) * d + t));
                    }
                    K8[((int64_t)h * Cp + slot) * d + t] = ck;
                    V8T[(((int64_t)h * n_blk + blk) * d + t) * 64 + j] = cv;
                }
            }
        }
    }
    return 0;
}

/*
 * Attention over the 8-bit cache: oracle_sparse_attn_fwd on the exact values of the E4M3 codes of K and V and of
 * the queries rounded to E4M3 (the kernel feeds both operands of the score product in that format); logits,
 * softmax and the weighted sum in fp64 as everywhere.  Q [H,n_q,d] (dtype), K8 / V8T as oracle_kv_to_fp8 writes
 * them, BK must be 64.
 */
int oracle_sparse_attn_fwd_fp8(const void *Q, int n_q, const uint8_t *K8, const uint8_t *V8T, const int32_t *cnt,
                               const int32_t *len, int H, int C, int d, int dtype, const int32_t *sel,
                               const int32_t *nsel, int BQ, int BK, int n_sel, double scale, double *O, double *lse) {
    if (!Q || !K8 || !V8T || BK != 64) return -1;
    const int n_blk = (C + 63) / 64;
    const int64_t Cp = (int64_t)n_blk * 64;
    float *Kf = malloc(sizeof(float) * (size_t)H * C * d);
    float *Vf = malloc(sizeof(float) * (size_t)H * C * d);
    float *Qf = malloc(sizeof(float) * (size_t)H * n_q * d);
    if (!Kf || !Vf || !Qf) {
        free(Kf);
        free(Vf);
        free(Qf);
        return -5;
    }
    for (int h = 0; h < H; ++h)
        for (int slot = 0; slot < C; ++slot)
            for (int t = 0; t < d; ++t) {
                Kf[((int64_t)h * C + slot) * d + t] = (float)fp8_value(K8[((int64_t)h * Cp + slot) * d + t]);
                Vf[((int64_t)h * C + slot) * d + t] =
                    (float)fp8_value(V8T[(((int64_t)h * n_blk + slot / 64) * d + t) * 64 + slot % 64]);
            }
    for (int64_t i = 0; i < (int64_t)H * n_q * d; ++i) Qf[i] = (float)fp8_value(fp8_code(load_f32(Q, dtype, i)));
    const int rc = oracle_sparse_attn_fwd(Qf, n_q, Kf, Vf, cnt, len, H, C, d, 0, sel, nsel, BQ, BK, n_sel, scale, O, lse);
    free(Kf);
    free(Vf);
    free(Qf);
    return rc;
}
