/*
 * PrefixKV CPU oracle -- TEST INFRASTRUCTURE, not a product path.
 *
 * A plain, slow, fp64 implementation of the five stages of the PrefixKV hot path, written from the
 * paper's definitions (Sec. 3.2 "Layer-wise KV Cache Importance Distribution", Sec. 3.3 "PrefixKV",
 * Eq. 1, Algorithm 1).  It shares no code with the HIP library and is only used by the tests, by
 * the smoke check and by the benchmark's cpu_baseline leg.
 *
 * Conventions: all pointers are host memory, arrays are dense row-major.  Inputs arrive as fp32
 * values that are already exactly representable in the storage dtype (the workload generator does
 * the rounding); all arithmetic below is fp64 unless a step says otherwise.
 *
 * OpenMP is used only across independent units (b,l,h), (b,l) or b; every reduction that crosses
 * units is done serially in a fixed order, so results do not depend on the thread count.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum { PKVO_NONFINITE = 1, PKVO_NEGATIVE = 2, PKVO_ZERO_LAYER = 4, PKVO_RANGE = 8 };

int pkvo_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---------------------------------------------------------------------------------------------
 * Stage 1 -- importance (Sec. 3.2).
 * a[m][n] = exp(scale*q_m.k_n) / sum_{j<=m} exp(scale*q_m.k_j)   for n <= m   (causal score matrix)
 * I[n]    = mean over the H query heads of sum_{m>=n} a[m][n]               (importance metric)
 * Query head h reads KV head h / (H/Hkv).  The paper's literal formula has scale = 1.
 * q [B,L,H,N,D], k [B,L,Hkv,N,D], scale [L] -> importance [B,L,N] (fp32 cast at the very end).
 * If lse_out != NULL it receives log(sum_j exp(scale*q_m.k_j)) per row, [B,L,H,N] fp64.
 * m_lo restricts the work to query rows m >= m_lo: since position n only receives attention from rows
 * m >= n, importance[.., n] is complete for every n >= m_lo (and NaN below), which lets a test check the
 * tail columns of a long prompt without paying for all rows.  m_lo = 0 computes everything.
 * ------------------------------------------------------------------------------------------- */
void pkvo_importance(int B, int L, int H, int Hkv, int N, int D, const float *q, const float *k,
                     const float *scale, float *importance, double *lse_out, int m_lo) {
    const int grp = H / Hkv;
    const long units = (long)B * L * H;
    double *colsum = (double *)calloc((size_t)units * N, sizeof(double));
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)N);
#pragma omp for schedule(dynamic, 1)
        for (long u = 0; u < units; ++u) {
            const int h = (int)(u % H);
            const int l = (int)((u / H) % L);
            const int b = (int)(u / ((long)H * L));
            const float *qh = q + (((size_t)b * L + l) * H + h) * (size_t)N * D;
            const float *kh = k + (((size_t)b * L + l) * Hkv + h / grp) * (size_t)N * D;
            double *cs = colsum + (size_t)u * N;
            const double sc = (double)scale[l];
            for (int m = m_lo; m < N; ++m) {
                double mx = -INFINITY;
                for (int n = 0; n <= m; ++n) {
                    double dot = 0.0;
                    for (int d = 0; d < D; ++d)
                        dot += (double)qh[(size_t)m * D + d] * (double)kh[(size_t)n * D + d];
                    s[n] = sc * dot;
                    if (s[n] > mx) mx = s[n];
                }
                double den = 0.0;
                for (int n = 0; n <= m; ++n) {
                    s[n] = exp(s[n] - mx);
                    den += s[n];
                }
                for (int n = 0; n <= m; ++n) cs[n] += s[n] / den;
                if (lse_out) lse_out[(size_t)u * N + m] = mx + log(den);
            }
        }
        free(s);
    }
    /* Average over heads, fixed order h = 0..H-1. */
    for (long bl = 0; bl < (long)B * L; ++bl)
        for (int n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int h = 0; h < H; ++h) acc += colsum[((size_t)bl * H + h) * N + n];
            importance[(size_t)bl * N + n] = n >= m_lo ? (float)(acc / (double)H) : NAN;
        }
    free(colsum);
}

/* ---------------------------------------------------------------------------------------------
 * Stage 2 -- priority sequence and cumulative priority (Sec. 3.2).
 * The priority sequence is the positions sorted by importance, descending; equal values keep the
 * lower position first (-0.0 counts as +0.0).  The normalised cumulative priority P^o is kept as an
 * exact integer pair (C_k, T): weight w = floor(importance * 2^36) as u64, C_k = sum of the first k
 * sorted weights, T = C_N, so P^{k/N} = C_k / T with no rounding anywhere.
 * ------------------------------------------------------------------------------------------- */
typedef struct {
    float v;
    int32_t pos;
} pkvo_item;

static int pkvo_item_cmp(const void *a, const void *b) {
    const pkvo_item *x = (const pkvo_item *)a, *y = (const pkvo_item *)b;
    if (x->v > y->v) return -1;
    if (x->v < y->v) return 1;
    return (x->pos > y->pos) - (x->pos < y->pos);
}

/* One layer.  Returns status bits; on a non-zero status the outputs are unspecified. */
int pkvo_sort_prefix_layer(int N, const float *imp, int32_t *order, uint64_t *cum, float *prefix) {
    int status = 0;
    for (int n = 0; n < N; ++n) {
        if (isnan(imp[n]) || isinf(imp[n])) status |= PKVO_NONFINITE;
        else if (imp[n] < 0.0f) status |= PKVO_NEGATIVE;
    }
    if (status) return status;
    pkvo_item *it = (pkvo_item *)malloc(sizeof(pkvo_item) * (size_t)N);
    for (int n = 0; n < N; ++n) {
        it[n].v = imp[n] == 0.0f ? 0.0f : imp[n]; /* folds -0.0 into +0.0 */
        it[n].pos = n;
    }
    qsort(it, (size_t)N, sizeof(pkvo_item), pkvo_item_cmp);
    const double two36 = 68719476736.0;
    const uint64_t lim = (uint64_t)1 << 53;
    uint64_t c = 0;
    for (int j = 0; j < N; ++j) {
        order[j] = it[j].pos;
        double wd = floor((double)it[j].v * two36);
        if (wd >= 9007199254740992.0) { status |= PKVO_RANGE; wd = 0.0; }
        c += (uint64_t)wd;
        if (c > lim) status |= PKVO_RANGE;
        cum[j] = c;
    }
    free(it);
    if (status) return status;
    if (c == 0) return PKVO_ZERO_LAYER;
    if (prefix)
        for (int j = 0; j < N; ++j) prefix[j] = (float)((double)cum[j] / (double)c);
    return 0;
}

/* Prefix length of one layer for threshold p (Sec. 3.3: R_l = min{o | P_l^o >= p}), in tokens:
 * the smallest k in 1..N with C_k >= p*T; p >= 1 keeps everything by definition. */
static int pkvo_layer_len(int N, const uint64_t *cum, double p) {
    if (p >= 1.0) return N;
    const double thr = p * (double)cum[N - 1];
    int k = 1;
    for (int j = 1; j <= N - 1; ++j)
        if ((double)cum[j - 1] < thr) ++k;
    return k;
}

typedef struct {
    uint64_t rem;
    int l;
} pkvo_rem;

static int pkvo_rem_desc(const void *a, const void *b) {
    const pkvo_rem *x = (const pkvo_rem *)a, *y = (const pkvo_rem *)b;
    if (x->rem != y->rem) return x->rem > y->rem ? -1 : 1;
    return (x->l > y->l) - (x->l < y->l);
}
static int pkvo_rem_asc(const void *a, const void *b) {
    const pkvo_rem *x = (const pkvo_rem *)a, *y = (const pkvo_rem *)b;
    if (x->rem != y->rem) return x->rem < y->rem ? -1 : 1;
    return (x->l > y->l) - (x->l < y->l);
}

/* Proportional rescale of per-layer weights to an exact token budget (Sec. 3.3, last paragraph: once
 * the search has stopped within its threshold, the configuration it found is brought to the target
 * budget by scaling): lengths[l] = weight[l]*budget/K
 * rounded down and clamped to [1,N] (K = sum of the weights), then the missing tokens go one per
 * layer in order of largest remainder (ties: lower layer), cyclically; a surplus is taken back in order
 * of smallest remainder.  Requires L < budget < L*N and K > 0. */
static void pkvo_rescale(int L, int N, const int64_t *weight, int64_t K, int64_t budget, int32_t *lengths) {
    pkvo_rem *r = (pkvo_rem *)malloc(sizeof(pkvo_rem) * (size_t)L);
    int64_t sum = 0;
    for (int l = 0; l < L; ++l) {
        const uint64_t num = (uint64_t)weight[l] * (uint64_t)budget;
        int64_t base = (int64_t)(num / (uint64_t)K);
        if (base < 1) base = 1;
        if (base > N) base = N;
        r[l].rem = num % (uint64_t)K;
        r[l].l = l;
        lengths[l] = (int32_t)base;
        sum += base;
    }
    int64_t dlt = budget - sum;
    if (dlt > 0) {
        qsort(r, (size_t)L, sizeof(pkvo_rem), pkvo_rem_desc);
        for (int i = 0; dlt > 0; i = (i + 1) % L)
            if (lengths[r[i].l] < N) { lengths[r[i].l] += 1; --dlt; }
    } else if (dlt < 0) {
        qsort(r, (size_t)L, sizeof(pkvo_rem), pkvo_rem_asc);
        for (int i = 0; dlt < 0; i = (i + 1) % L)
            if (lengths[r[i].l] > 1) { lengths[r[i].l] -= 1; ++dlt; }
    }
    free(r);
}

/* ---------------------------------------------------------------------------------------------
 * Stage 3 -- Algorithm 1 (binary search for the retention ratio p) for ONE sequence, followed by
 * the rescale to the exact budget of Sec. 3.3's last paragraph.
 * cum [L,N]; budget/tol in tokens.  Outputs lengths[L], *p, *iters, *raw_total (sum of lengths of
 * the last evaluated p, before scaling).
 * ------------------------------------------------------------------------------------------- */
void pkvo_search(int L, int N, const uint64_t *cum, int64_t budget, int64_t tol, int max_iters,
                 int fixup, int32_t *lengths, double *p_out, int32_t *iters_out,
                 int64_t *raw_total_out) {
    if (budget <= L) { /* nothing below one vector per layer: o starts at 1/N */
        for (int l = 0; l < L; ++l) lengths[l] = 1;
        *p_out = 0.0; *iters_out = 0; *raw_total_out = L;
        return;
    }
    if (budget >= (int64_t)L * N) { /* budget of 100%: no compression */
        for (int l = 0; l < L; ++l) lengths[l] = N;
        *p_out = 1.0; *iters_out = 0; *raw_total_out = (int64_t)L * N;
        return;
    }
    double p1 = 0.0, p2 = 1.0, p = 0.5;
    int64_t K = 0;
    int iters = 0;
    for (int it = 1; it <= max_iters; ++it) {
        const double mid = 0.5 * (p1 + p2);
        if (mid == p1 || mid == p2) break; /* interval cannot shrink any more */
        p = mid;
        K = 0;
        for (int l = 0; l < L; ++l) {
            lengths[l] = pkvo_layer_len(N, cum + (size_t)l * N, p);
            K += lengths[l];
        }
        iters = it;
        const int64_t delta = K - budget;
        if (llabs(delta) <= tol) break;
        if (delta < 0) p1 = p; else p2 = p;
    }
    *p_out = p; *iters_out = iters; *raw_total_out = K;
    if (!fixup || K == budget) return;

    int64_t *wgt = (int64_t *)malloc(sizeof(int64_t) * (size_t)L);
    for (int l = 0; l < L; ++l) wgt[l] = lengths[l];
    pkvo_rescale(L, N, wgt, K, budget, lengths);
    free(wgt);
}

/* Offline estimation of the global prefix configuration (Sec. 3.3, last paragraph: the configuration is
 * derived from a few random samples and then adopted for every input, which avoids the online search).
 * The paper does not give the aggregation rule; this reading averages the per-sample ratios R_l, i.e.
 * weights layer l by the sum of its lengths over the S samples, and rescales those weights to the
 * budget of the deployed prompt length N with the same largest-remainder rule.
 * sample_lengths [S,L] (all samples share one prompt length) -> lengths [L].
 * budget <= L gives all 1, budget >= L*N all N; an all-zero sample set gives all 0. */
void pkvo_offline_config(int S, int L, int N, const int32_t *sample_lengths, int64_t budget,
                         int32_t *lengths) {
    int64_t *wgt = (int64_t *)calloc((size_t)L, sizeof(int64_t));
    int64_t K = 0;
    for (int s = 0; s < S; ++s)
        for (int l = 0; l < L; ++l) { wgt[l] += sample_lengths[(size_t)s * L + l]; K += sample_lengths[(size_t)s * L + l]; }
    if (K == 0) { for (int l = 0; l < L; ++l) lengths[l] = 0; }
    else if (budget <= L) { for (int l = 0; l < L; ++l) lengths[l] = 1; }
    else if (budget >= (int64_t)L * N) { for (int l = 0; l < L; ++l) lengths[l] = N; }
    else pkvo_rescale(L, N, wgt, K, budget, lengths);
    free(wgt);
}

/* Stages 2+3 for a batch: importance [B,L,N] -> order, cum, prefix (may be NULL), lengths [B,L],
 * p [B], iters [B], raw_total [B], status [B].  A sequence with a non-zero status gets
 * lengths = 0, p = 0, iters = 0, raw_total = 0. */
void pkvo_select(int B, int L, int N, const float *importance, int64_t budget, int64_t tol,
                 int max_iters, int fixup, int32_t *order, uint64_t *cum, float *prefix,
                 int32_t *lengths, double *p, int32_t *iters, int64_t *raw_total, int32_t *status) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        int st = 0;
        for (int l = 0; l < L; ++l) {
            const size_t o = ((size_t)b * L + l) * N;
            st |= pkvo_sort_prefix_layer(N, importance + o, order + o, cum + o,
                                         prefix ? prefix + o : NULL);
        }
        status[b] = st;
        if (st) {
            for (int l = 0; l < L; ++l) lengths[(size_t)b * L + l] = 0;
            p[b] = 0.0; iters[b] = 0; raw_total[b] = 0;
        } else {
            pkvo_search(L, N, cum + (size_t)b * L * N, budget, tol, max_iters, fixup,
                        lengths + (size_t)b * L, p + b, iters + b, raw_total + b);
        }
    }
}

/* ---------------------------------------------------------------------------------------------
 * Stage 4a -- compaction (Sec. 3.2: the top R_l proportion is retained in each head of layer l).
 * The kept set of (b,l) is the first lengths[b,l] entries of its priority sequence; it is stored in
 * ascending original position.  Ragged layout: segment (b,l) starts at token offset seg_off[b,l]
 * (exclusive scan of caps = lengths + decode_capacity in (b,l) order) and holds [Hkv][cap][D].
 * kc/vc must hold sum(caps)*Hkv*D floats; slots beyond the kept ones are left untouched.
 * ------------------------------------------------------------------------------------------- */
static int pkvo_i32_cmp(const void *a, const void *b) {
    const int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

void pkvo_compact(int B, int L, int Hkv, int N, int D, const float *k, const float *v,
                  const int32_t *order, const int32_t *lengths, int decode_capacity,
                  int64_t *seg_off, int32_t *caps, float *kc, float *vc, int32_t *kept_pos,
                  int32_t *lens) {
    int64_t off = 0;
    for (long bl = 0; bl < (long)B * L; ++bl) {
        caps[bl] = lengths[bl] + decode_capacity;
        seg_off[bl] = off;
        off += caps[bl];
        lens[bl] = lengths[bl];
    }
#pragma omp parallel for schedule(dynamic, 1)
    for (long bl = 0; bl < (long)B * L; ++bl) {
        const int kl = lengths[bl];
        const int cap = caps[bl];
        int32_t *kp = kept_pos + seg_off[bl];
        memcpy(kp, order + (size_t)bl * N, sizeof(int32_t) * (size_t)kl);
        qsort(kp, (size_t)kl, sizeof(int32_t), pkvo_i32_cmp);
        for (int h = 0; h < Hkv; ++h) {
            const float *ksrc = k + ((size_t)bl * Hkv + h) * (size_t)N * D;
            const float *vsrc = v + ((size_t)bl * Hkv + h) * (size_t)N * D;
            float *kdst = kc + ((size_t)seg_off[bl] * Hkv + (size_t)h * cap) * D;
            float *vdst = vc + ((size_t)seg_off[bl] * Hkv + (size_t)h * cap) * D;
            for (int j = 0; j < kl; ++j) {
                memcpy(kdst + (size_t)j * D, ksrc + (size_t)kp[j] * D, sizeof(float) * (size_t)D);
                memcpy(vdst + (size_t)j * D, vsrc + (size_t)kp[j] * D, sizeof(float) * (size_t)D);
            }
        }
    }
}

/* Round-to-nearest-even to bfloat16, returned as the fp32 value it represents. */
static float pkvo_round_bf16(double x) {
    float f = (float)x;
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return f; /* NaN */
    u += 0x7fffu + ((u >> 16) & 1u);
    u &= 0xffff0000u;
    memcpy(&f, &u, 4);
    return f;
}

/* ---------------------------------------------------------------------------------------------
 * Stage 4b -- one decode step for layers [l0,l1) (Sec. 3.1: the newest token's query interacts
 * with the cached KV vectors).  If k_new/v_new are given they are appended at slot lens[b,l] first
 * and lens is incremented.  o = softmax_j(scale_l * q.Kc_j) . Vc over the lens slots.
 * q [B,L,H,D], k_new/v_new [B,L,Hkv,D], out [B,L,H,D] (rounded to bf16 if out_bf16).
 * Returns -1 if an append would exceed a segment's capacity (nothing is modified then).
 * ------------------------------------------------------------------------------------------- */
int pkvo_decode_attn(int B, int L, int H, int Hkv, int D, int l0, int l1, const float *q,
                     const float *k_new, const float *v_new, const float *scale, float *kc,
                     float *vc, const int64_t *seg_off, const int32_t *caps, int32_t *lens,
                     float *out, int out_bf16) {
    const int grp = H / Hkv;
    if (k_new)
        for (int b = 0; b < B; ++b)
            for (int l = l0; l < l1; ++l)
                if (lens[b * L + l] + 1 > caps[b * L + l]) return -1;
#pragma omp parallel for schedule(dynamic, 1) collapse(2)
    for (int b = 0; b < B; ++b)
        for (int l = l0; l < l1; ++l) {
            const long bl = (long)b * L + l;
            const int cap = caps[bl];
            int len = lens[bl];
            if (k_new) {
                for (int h = 0; h < Hkv; ++h) {
                    const size_t dst = ((size_t)seg_off[bl] * Hkv + (size_t)h * cap + len) * D;
                    memcpy(kc + dst, k_new + ((size_t)bl * Hkv + h) * D, sizeof(float) * (size_t)D);
                    memcpy(vc + dst, v_new + ((size_t)bl * Hkv + h) * D, sizeof(float) * (size_t)D);
                }
                len += 1;
                lens[bl] = len;
            }
            double *s = (double *)malloc(sizeof(double) * (size_t)(len > 0 ? len : 1));
            for (int h = 0; h < H; ++h) {
                const float *qh = q + ((size_t)bl * H + h) * D;
                const size_t base = ((size_t)seg_off[bl] * Hkv + (size_t)(h / grp) * cap) * D;
                float *oh = out + ((size_t)bl * H + h) * D;
                if (len == 0) { /* empty cache: defined as a zero output */
                    for (int d = 0; d < D; ++d) oh[d] = 0.0f;
                    continue;
                }
                double mx = -INFINITY;
                for (int j = 0; j < len; ++j) {
                    double dot = 0.0;
                    for (int d = 0; d < D; ++d)
                        dot += (double)qh[d] * (double)kc[base + (size_t)j * D + d];
                    s[j] = (double)scale[l] * dot;
                    if (s[j] > mx) mx = s[j];
                }
                double den = 0.0;
                for (int j = 0; j < len; ++j) { s[j] = exp(s[j] - mx); den += s[j]; }
                for (int d = 0; d < D; ++d) {
                    double acc = 0.0;
                    for (int j = 0; j < len; ++j)
                        acc += s[j] * (double)vc[base + (size_t)j * D + d];
                    acc /= den;
                    oh[d] = out_bf16 ? pkvo_round_bf16(acc) : (float)acc;
                }
            }
            free(s);
        }
    return 0;
}

/* ---------------------------------------------------------------------------------------------
 * Decode step with ratio maintenance (Sec. 3.1 last sentences and Fig. 3 caption: during decoding the
 * vectors at a fixed distance to the latest generated token are pruned so that the global prefix
 * configuration is maintained).  The paper gives neither the distance nor the bookkeeping; this reading:
 *   - R_l = base_lens[b,l] / N is the layer's retention ratio found after prefill;
 *   - after decode step t (1-based, sequence length N+t) the layer aims at
 *       target(t) = max(1, round_half_up(R_l * (N+t))) cached entries;
 *   - step t first stores the new token; then the token generated d steps earlier (token t-d, the one
 *     at distance d from the newest) is decided once and for all: it stays for ever if the cache with
 *     it is within the target, else it is pruned; for t <= d nothing is decided (the token at distance
 *     d belongs to the prompt, whose selection the prefix configuration already made);
 *   - the d newest tokens are always cached; the query of step t attends to the cache after pruning.
 * Physical layout of a segment of `cap` slots: slots [0, lens) are the permanent entries (kept prompt
 * positions, then survivors in the order they were decided), the LAST d+1 slots are a ring: token j sits
 * in ring slot (j-1) mod (d+1), so the token decided in step t occupies the slot the next token will
 * overwrite.  lens[b,l] counts permanent entries only.  kept_pos holds the sequence position of every
 * live slot (prompt positions 0..N-1, decode token j at N+j-1), -1 for a pruned ring slot.
 * Returns -1 (nothing modified) if d < 1, a ring does not fit behind the kept prompt entries, or a
 * survivor would not fit in front of the ring.
 * ------------------------------------------------------------------------------------------- */
static int64_t pkvo_target(int64_t k_l, int64_t N, int64_t t) {
    const int64_t r = (2 * k_l * (N + t) + N) / (2 * N);
    return r < 1 ? 1 : r;
}

int pkvo_decode_attn_evict(int B, int L, int H, int Hkv, int N, int D, int l0, int l1, const float *q,
                           const float *k_new, const float *v_new, const float *scale, float *kc,
                           float *vc, int32_t *kept_pos, const int64_t *seg_off, const int32_t *caps,
                           const int32_t *base_lens, int32_t *lens, int t, int d, float *out,
                           int out_bf16) {
    const int grp = H / Hkv;
    if (d < 1 || t < 1) return -1;
    for (int b = 0; b < B; ++b)
        for (int l = l0; l < l1; ++l) {
            const long bl = (long)b * L + l;
            const int ring0 = caps[bl] - (d + 1);
            if (ring0 < base_lens[bl] || lens[bl] > ring0) return -1;
            if (t > d && lens[bl] + d + 1 <= pkvo_target(base_lens[bl], N, t) && lens[bl] >= ring0) return -1;
        }
#pragma omp parallel for schedule(dynamic, 1) collapse(2)
    for (int b = 0; b < B; ++b)
        for (int l = l0; l < l1; ++l) {
            const long bl = (long)b * L + l;
            const int cap = caps[bl];
            const int ring0 = cap - (d + 1);
            int perm = lens[bl];
            int32_t *kp = kept_pos + seg_off[bl];
            /* 1. store token t in its ring slot */
            const int ns = ring0 + (t - 1) % (d + 1);
            for (int h = 0; h < Hkv; ++h) {
                const size_t dst = ((size_t)seg_off[bl] * Hkv + (size_t)h * cap + ns) * D;
                memcpy(kc + dst, k_new + ((size_t)bl * Hkv + h) * D, sizeof(float) * (size_t)D);
                memcpy(vc + dst, v_new + ((size_t)bl * Hkv + h) * D, sizeof(float) * (size_t)D);
            }
            kp[ns] = N + t - 1;
            /* 2. decide token t-d */
            if (t > d) {
                const int cs = ring0 + t % (d + 1);
                if (perm + d + 1 <= pkvo_target(base_lens[bl], N, t)) {
                    for (int h = 0; h < Hkv; ++h) {
                        const size_t sb = ((size_t)seg_off[bl] * Hkv + (size_t)h * cap) * D;
                        memcpy(kc + sb + (size_t)perm * D, kc + sb + (size_t)cs * D, sizeof(float) * (size_t)D);
                        memcpy(vc + sb + (size_t)perm * D, vc + sb + (size_t)cs * D, sizeof(float) * (size_t)D);
                    }
                    kp[perm] = kp[cs];
                    perm += 1;
                }
                /* survivor or not, the ring slot no longer holds a cached entry */
                for (int h = 0; h < Hkv; ++h) {
                    const size_t sb = ((size_t)seg_off[bl] * Hkv + (size_t)h * cap + cs) * D;
                    for (int x = 0; x < D; ++x) { kc[sb + x] = NAN; vc[sb + x] = NAN; }
                }
                kp[cs] = -1;
                lens[bl] = perm;
            }
            /* 3. attention of the new query over the live slots: permanent entries, then ring */
            int *slot = (int *)malloc(sizeof(int) * (size_t)(perm + d + 1));
            int n = 0;
            for (int j = 0; j < perm; ++j) slot[n++] = j;
            for (int j = 0; j <= d; ++j)
                if (kp[ring0 + j] >= 0) slot[n++] = ring0 + j; /* stored and not yet decided */
            double *s = (double *)malloc(sizeof(double) * (size_t)n);
            for (int h = 0; h < H; ++h) {
                const float *qh = q + ((size_t)bl * H + h) * D;
                const size_t base = ((size_t)seg_off[bl] * Hkv + (size_t)(h / grp) * cap) * D;
                float *oh = out + ((size_t)bl * H + h) * D;
                double mx = -INFINITY;
                for (int j = 0; j < n; ++j) {
                    double dot = 0.0;
                    for (int x = 0; x < D; ++x)
                        dot += (double)qh[x] * (double)kc[base + (size_t)slot[j] * D + x];
                    s[j] = (double)scale[l] * dot;
                    if (s[j] > mx) mx = s[j];
                }
                double den = 0.0;
                for (int j = 0; j < n; ++j) { s[j] = exp(s[j] - mx); den += s[j]; }
                for (int x = 0; x < D; ++x) {
                    double acc = 0.0;
                    for (int j = 0; j < n; ++j)
                        acc += s[j] * (double)vc[base + (size_t)slot[j] * D + x];
                    acc /= den;
                    oh[x] = out_bf16 ? pkvo_round_bf16(acc) : (float)acc;
                }
            }
            free(s);
            free(slot);
        }
    return 0;
}

/* ---------------------------------------------------------------------------------------------
 * Gini coefficient of a layer's priority sequence (Sec. 4.3, "Relation between KV cache size and
 * importance distribution": layers with a more concentrated importance distribution, i.e. a higher
 * Gini coefficient, get smaller caches).  With the Lorenz curve through the points
 * (j/N, share of the j smallest weights) and the trapezoid rule, G = 1 - 2 * area under the curve.
 * On the exact fixed-point cumulative sums C_k of the descending sequence (C_N = T) this is
 *   G = (2 * (C_1 + ... + C_N) / T - N - 1) / N,
 * 0 for a flat layer and (N-1)/N when one position holds everything.  T = 0 gives 0.
 * cum [B*L][N] u64 -> gini [B*L] f64.
 * ------------------------------------------------------------------------------------------- */
void pkvo_gini(long segs, int N, const uint64_t *cum, double *gini) {
    for (long s = 0; s < segs; ++s) {
        const uint64_t *c = cum + (size_t)s * N;
        unsigned __int128 S = 0;
        for (int k = 0; k < N; ++k) S += c[k];
        const double T = (double)c[N - 1];
        gini[s] = T > 0.0 ? (2.0 * ((double)S / T) - (double)N - 1.0) / (double)N : 0.0;
    }
}

/* ---------------------------------------------------------------------------------------------
 * Cache merging by positional distance (Sec. 4.3, "Eviction or merging", the variant called
 * "Position": matching metric c^{mn} = -|m - n|).  Every pruned position m of a layer is matched to
 * the retained position n with the largest metric, i.e. the nearest one (a pruned position half way
 * between two retained ones goes to the lower: the first maximum), and every retained vector is
 * replaced by the average of itself and the pruned vectors matched to it; keys and values of all
 * heads alike.  Works in place on a cache produced by pkvo_compact: slot j of segment (b,l) holds
 * position kept_pos[j]; only the first lens[b,l] slots are touched.  The average is taken in fp64
 * and, if storage_bf16, rounded to bfloat16 like every stored vector.
 * k, v [B,L,Hkv,N,D] are the uncompressed tensors.
 * ------------------------------------------------------------------------------------------- */
void pkvo_merge_position(int B, int L, int Hkv, int N, int D, const float *k, const float *v,
                         const int64_t *seg_off, const int32_t *caps, const int32_t *kept_pos,
                         const int32_t *lens, float *kc, float *vc, int storage_bf16) {
#pragma omp parallel for schedule(dynamic, 1)
    for (long bl = 0; bl < (long)B * L; ++bl) {
        const int n = lens[bl], cap = caps[bl];
        if (n <= 0) continue;
        const int32_t *kp = kept_pos + seg_off[bl];
        int *match = (int *)malloc(sizeof(int) * (size_t)N); /* slot every position is averaged into */
        for (int m = 0; m < N; ++m) {
            int best = 0;
            long bestc = -labs((long)m - kp[0]);
            for (int j = 1; j < n; ++j) {
                const long c = -labs((long)m - kp[j]);
                if (c > bestc) { bestc = c; best = j; } /* first maximum: slots ascend with position */
            }
            match[m] = best;
        }
        double *acc = (double *)malloc(sizeof(double) * (size_t)D);
        for (int h = 0; h < Hkv; ++h)
            for (int which = 0; which < 2; ++which) {
                const float *src = (which ? v : k) + ((size_t)bl * Hkv + h) * (size_t)N * D;
                float *dst = (which ? vc : kc) + ((size_t)seg_off[bl] * Hkv + (size_t)h * cap) * D;
                for (int j = 0; j < n; ++j) {
                    int cnt = 0;
                    for (int x = 0; x < D; ++x) acc[x] = 0.0;
                    for (int m = 0; m < N; ++m)
                        if (match[m] == j) {
                            ++cnt;
                            for (int x = 0; x < D; ++x) acc[x] += (double)src[(size_t)m * D + x];
                        }
                    for (int x = 0; x < D; ++x) {
                        const double mean = acc[x] / (double)cnt;
                        dst[(size_t)j * D + x] = storage_bf16 ? pkvo_round_bf16(mean) : (float)mean;
                    }
                }
            }
        free(acc);
        free(match);
    }
}

/* ---------------------------------------------------------------------------------------------
 * Cache merging by feature similarity (Sec. 4.3, "Eviction or merging", the variant called "Feature":
 * matching metric c^{mn} = cosine of the pruned vector m and the retained vector n).  The paper
 * describes the operation on the key vectors of one head and says that values and the other heads
 * are treated the same way; the reading taken here is the literal one: every (head, tensor) pair is
 * merged on its own, with the cosine of ITS vectors (keys by key similarity, values by value
 * similarity).  A vector of norm zero has cosine 0 with everything.
 *
 * pkvo_feature_match: x [B,L,Hkv,N,D] (keys OR values, uncompressed); the retained set of (b,l) is
 * kept_pos[seg_off .. +lens) (ascending positions).  match [B,L,Hkv,N] gets, for a pruned position,
 * the slot of the retained vector with the largest cosine (first maximum = lowest position), for a
 * retained position -1; best (may be NULL) gets that largest cosine (1 for retained positions).
 * pkvo_match_cosine: the cosine of every pruned position with the slot a GIVEN assignment names
 * (what a test needs to accept a different but equally good choice on a near tie).
 * pkvo_merge_by_match: slot j of the compressed tensor xc := average of the retained vector and of all
 * pruned vectors assigned to it, in fp64, rounded to bfloat16 if storage_bf16.
 * ------------------------------------------------------------------------------------------- */
static double pkvo_cosine(const float *a, const float *b, int D) {
    double dot = 0.0, na = 0.0, nb = 0.0;
    for (int x = 0; x < D; ++x) {
        dot += (double)a[x] * (double)b[x];
        na += (double)a[x] * (double)a[x];
        nb += (double)b[x] * (double)b[x];
    }
    return (na > 0.0 && nb > 0.0) ? dot / (sqrt(na) * sqrt(nb)) : 0.0;
}

void pkvo_feature_match(int B, int L, int Hkv, int N, int D, const float *x, const int64_t *seg_off,
                        const int32_t *kept_pos, const int32_t *lens, int32_t *match, double *best) {
#pragma omp parallel for schedule(dynamic, 1)
    for (long u = 0; u < (long)B * L * Hkv; ++u) {
        const long bl = u / Hkv;
        const int n = lens[bl];
        const int32_t *kp = kept_pos + seg_off[bl];
        const float *xh = x + (size_t)u * N * D;
        int32_t *mt = match + (size_t)u * N;
        for (int m = 0; m < N; ++m) {
            int arg = 0;
            double top = -INFINITY;
            for (int j = 0; j < n; ++j) {
                const double c = pkvo_cosine(xh + (size_t)m * D, xh + (size_t)kp[j] * D, D);
                if (c > top) { top = c; arg = j; }
            }
            mt[m] = arg;
            if (best) best[(size_t)u * N + m] = top;
        }
        for (int j = 0; j < n; ++j) {
            mt[kp[j]] = -1;
            if (best) best[(size_t)u * N + kp[j]] = 1.0;
        }
    }
}

void pkvo_match_cosine(int B, int L, int Hkv, int N, int D, const float *x, const int64_t *seg_off,
                       const int32_t *kept_pos, const int32_t *match, double *cosine) {
    for (long u = 0; u < (long)B * L * Hkv; ++u) {
        const int32_t *kp = kept_pos + seg_off[u / Hkv];
        const float *xh = x + (size_t)u * N * D;
        for (int m = 0; m < N; ++m) {
            const int j = match[(size_t)u * N + m];
            cosine[(size_t)u * N + m] = j < 0 ? 1.0 : pkvo_cosine(xh + (size_t)m * D, xh + (size_t)kp[j] * D, D);
        }
    }
}

void pkvo_merge_by_match(int B, int L, int Hkv, int N, int D, const float *x, const int64_t *seg_off,
                         const int32_t *caps, const int32_t *kept_pos, const int32_t *lens,
                         const int32_t *match, float *xc, int storage_bf16) {
#pragma omp parallel for schedule(dynamic, 1)
    for (long u = 0; u < (long)B * L * Hkv; ++u) {
        const long bl = u / Hkv;
        const int h = (int)(u % Hkv), n = lens[bl];
        const int32_t *kp = kept_pos + seg_off[bl];
        const float *xh = x + (size_t)u * N * D;
        const int32_t *mt = match + (size_t)u * N;
        float *dst = xc + ((size_t)seg_off[bl] * Hkv + (size_t)h * caps[bl]) * D;
        double *acc = (double *)malloc(sizeof(double) * (size_t)D);
        for (int j = 0; j < n; ++j) {
            int cnt = 1;
            for (int d = 0; d < D; ++d) acc[d] = (double)xh[(size_t)kp[j] * D + d];
            for (int m = 0; m < N; ++m)
                if (mt[m] == j) {
                    ++cnt;
                    for (int d = 0; d < D; ++d) acc[d] += (double)xh[(size_t)m * D + d];
                }
            for (int d = 0; d < D; ++d) {
                const double mean = acc[d] / (double)cnt;
                dst[(size_t)j * D + d] = storage_bf16 ? pkvo_round_bf16(mean) : (float)mean;
            }
        }
        free(acc);
    }
}

/* ---------------------------------------------------------------------------------------------
 * Causal prefill attention of one prompt (Sec. 3.1: the prefill phase computes the attention of all
 * prompt tokens; Sec. 3.2 builds the importance from the same score matrix a_l^{i,m,n}).
 *   out[m] = sum_{n<=m} a[m][n] * v[n],  a[m][n] = exp(scale*q_m.k_n) / sum_{j<=m} exp(scale*q_m.k_j)
 *   lse[m] = log sum_{j<=m} exp(scale*q_m.k_j)      (what the importance stage accepts from its caller)
 * q [B,L,H,N,D], k/v [B,L,Hkv,N,D] -> out [B,L,H,N,D] (rounded to bf16 if out_bf16), lse [B,L,H,N] f64.
 * ------------------------------------------------------------------------------------------- */
void pkvo_prefill_attn(int B, int L, int H, int Hkv, int N, int D, const float *q, const float *k,
                       const float *v, const float *scale, float *out, double *lse, int out_bf16) {
    const int grp = H / Hkv;
    const long units = (long)B * L * H;
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)N);
#pragma omp for schedule(dynamic, 1)
        for (long u = 0; u < units; ++u) {
            const int h = (int)(u % H);
            const int l = (int)((u / H) % L);
            const long bl = u / H;
            const float *qh = q + (size_t)u * N * D;
            const float *kh = k + ((size_t)bl * Hkv + h / grp) * (size_t)N * D;
            const float *vh = v + ((size_t)bl * Hkv + h / grp) * (size_t)N * D;
            for (int m = 0; m < N; ++m) {
                double mx = -INFINITY;
                for (int n = 0; n <= m; ++n) {
                    double dot = 0.0;
                    for (int d = 0; d < D; ++d) dot += (double)qh[(size_t)m * D + d] * (double)kh[(size_t)n * D + d];
                    s[n] = (double)scale[l] * dot;
                    if (s[n] > mx) mx = s[n];
                }
                double den = 0.0;
                for (int n = 0; n <= m; ++n) { s[n] = exp(s[n] - mx); den += s[n]; }
                lse[(size_t)u * N + m] = mx + log(den);
                for (int d = 0; d < D; ++d) {
                    double acc = 0.0;
                    for (int n = 0; n <= m; ++n) acc += s[n] * (double)vh[(size_t)n * D + d];
                    acc /= den;
                    out[((size_t)u * N + m) * D + d] = out_bf16 ? pkvo_round_bf16(acc) : (float)acc;
                }
            }
        }
        free(s);
    }
}
