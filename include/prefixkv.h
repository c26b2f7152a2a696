/*
 * prefixkv.h -- C ABI of the MI355X (gfx950) PrefixKV hot-path library.
 *
 * PrefixKV (arXiv 2412.03409) compresses the KV cache of a decoder after prefill: every cached
 * position of layer l gets an importance (Sec. 3.2), positions are ranked per layer, and ONE
 * retention ratio p, found by the binary search of Algorithm 1 (Sec. 3.3, Eq. 1), decides how long
 * a prefix of each layer's ranking is kept so that all layers together meet a KV budget.
 *
 * General rules for every entry point
 *   - Pointers marked [dev] are device (HBM) memory OWNED BY THE CALLER; [host] are host memory.
 *     The library never allocates, frees or synchronises.  All work is enqueued on `stream`
 *     (a hipStream_t passed as void*; NULL = the default stream) and may still be running when the
 *     call returns.  Scratch space comes from the caller: `ws` [dev], `ws_bytes` >= the value of
 *     prefixkv_workspace_bytes() for the same arguments; its contents are undefined afterwards
 *     and nothing is carried in it from one call to the next.
 *   - The return value reports ARGUMENT errors synchronously (pkv_status); nothing is enqueued
 *     when it is non-zero.  Data-dependent problems are reported through device status words.
 *   - Layouts are row-major with the head dimension D contiguous.  Where strides are given they
 *     are in ELEMENTS.  D is 64 or 128, H % Hkv == 0, 1 <= L <= 64, 1 <= N <= 8192, B >= 1.
 *   - Calls that use the same workspace or the same output buffers must be ordered by the
 *     caller (same stream, or events).  The library keeps no state between calls (apart from the
 *     device's compute-unit count and, for prefixkv_select_static, the address of its built-in
 *     scratch array, each looked up once per device).
 */
#ifndef PREFIXKV_H
#define PREFIXKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PKV_OK = 0,
    PKV_ERR_NULL = 1,        /* a required pointer is NULL */
    PKV_ERR_DIM = 2,         /* a dimension is out of the supported range */
    PKV_ERR_DTYPE = 3,       /* unknown dtype */
    PKV_ERR_STRIDE = 4,      /* stride not a multiple of 8 elements (16-byte rows needed) or negative */
    PKV_ERR_WORKSPACE = 5,   /* ws is NULL or ws_bytes too small */
    PKV_ERR_BUDGET = 6,      /* budget_tokens < 1, tol_tokens < 0 or max_iters < 1 */
    PKV_ERR_UNSUPPORTED = 7, /* valid request this build has no kernel for */
    PKV_ERR_HIP = 8          /* a launch failed; see hipGetLastError */
} pkv_status;

/* bits of the per-sequence device status word written by prefixkv_select */
enum {
    PKV_DEV_NONFINITE = 1,  /* importance holds NaN or Inf */
    PKV_DEV_NEGATIVE = 2,   /* importance holds a negative value (-0.0 is accepted as 0) */
    PKV_DEV_ZERO_LAYER = 4, /* some layer's fixed-point weights are all zero */
    PKV_DEV_RANGE = 8       /* a layer's importance sums to more than 2^17 */
};

typedef enum { PKV_F32 = 0, PKV_BF16 = 1 } pkv_dtype;

/* B sequences, L layers, H query heads, Hkv key/value heads, N prompt positions, head dim D;
 * dtype is the storage type of Q/K/V, of the compressed cache and of the attention output. */
typedef struct { int32_t B, L, H, Hkv, N, D; int32_t dtype; } pkv_shape;

/* Element strides of a [B, L, heads, N, D] tensor (D-stride is 1). */
typedef struct { int64_t b, l, h, n; } pkv_strides;

typedef void *pkv_stream; /* hipStream_t */

int prefixkv_version(void);
const char *prefixkv_status_string(int status);

/* Workspace bytes for op = PKV_OP_*.  `has_lse` (PKV_OP_IMPORTANCE only) = the caller will pass
 * its own lse.  Returns 0 for invalid arguments and for stages that need no scratch (compaction;
 * decode attention unless several query heads share a KV head in a bf16 cache): ws may then be NULL. */
enum { PKV_OP_IMPORTANCE = 0, PKV_OP_SELECT = 1, PKV_OP_COMPACT = 2, PKV_OP_DECODE = 3, PKV_OP_MERGE_FEATURE = 4 };
size_t prefixkv_workspace_bytes(int op, const pkv_shape *shape, int has_lse);

/* ---- Stage 1: KV importance (Sec. 3.2, the causal score matrix a_l^{i,m,n} and the importance
 * metric I_l^n = Average_i(sum_m a_l^{i,m,n})).
 *   importance[b,l,n] = (1/H) * sum_h sum_{m>=n} softmax_{j<=m}(scale[l] * q[b,l,h,m,:].k[b,l,g(h),j,:])[n]
 * with g(h) = h / (H/Hkv).  The paper's formula has no logit scale (scale = 1); a model passes its
 * own, usually 1/sqrt(D).
 *   q [dev] [B,L,H,N,D] with strides qs;  k [dev] [B,L,Hkv,N,D] with strides ks  (shape->dtype)
 *   scale [dev] fp32 [L]
 *   lse [dev] fp32 [B,L,H,N] = log sum_{j<=m} exp(scale*q_m.k_j) of every causal row if the caller
 *       already has it from its prefill attention, or NULL: it is then computed here (a first sweep over
 *       the keys inside the same kernel).
 *   importance [dev] fp32 [B,L,N], out (dense).
 * bf16 inputs use bf16 MFMA with fp32 accumulation; exp and all sums are fp32. */
int prefixkv_importance(const pkv_shape *shape, const void *q, pkv_strides qs, const void *k,
                        pkv_strides ks, const float *scale, const float *lse, float *importance,
                        void *ws, size_t ws_bytes, pkv_stream stream);

/* ---- The step before the path: causal prefill attention that hands its row log-sum-exp to stage 1
 * (Sec. 3.1: the prefill phase attends over the whole prompt; Sec. 3.2 defines the importance on the
 * same score matrix, so a prefill kernel that keeps lse saves stage 1 one of its two sweeps over the keys).
 *   out[b,l,h,m,:] = sum_{n<=m} softmax_{j<=m}(scale[l] * q_m.k_j)[n] * v[b,l,g(h),n,:]
 *   lse[b,l,h,m]   = log sum_{j<=m} exp(scale[l] * q_m.k_j)         (natural log, fp32)
 * bf16 storage only (PKV_ERR_UNSUPPORTED otherwise); both products on bf16 MFMA with fp32 accumulation,
 * probabilities rounded to bf16 for the second product, fp32 softmax.
 *   q [dev] [B,L,H,N,D] strides qs;  k, v [dev] [B,L,Hkv,N,D] strides ks, vs;  scale [dev] fp32 [L]
 *   out [dev] bf16 [B,L,H,N,D] dense;  lse [dev] fp32 [B,L,H,N] dense: pass it as `lse` to
 *   prefixkv_importance.  No workspace. */
int prefixkv_prefill_attn(const pkv_shape *shape, const void *q, pkv_strides qs, const void *k,
                          pkv_strides ks, const void *v, pkv_strides vs, const float *scale,
                          void *out, float *lse, pkv_stream stream);

/* ---- Stages 2+3: priority sequences, cumulative priority and the global search (Sec. 3.2 for
 * the normalised, sorted, cumulated importance P_l^o; Sec. 3.3, Eq. 1 and Algorithm 1 for p).
 * Per sequence b and layer l:
 *   order[b,l,:]  positions sorted by importance descending, equal values by ascending position
 *   cum[b,l,k-1]  C_k = sum of the first k sorted fixed-point weights, weight = floor(imp * 2^36)
 *                 (exact integers; the cumulative priority of a prefix of k is C_k / C_N)
 *   prefix        (float)(C_k / C_N), informational, may be NULL
 * Per sequence b: Algorithm 1 on p in [0,1]; the prefix length of layer l at p is the smallest
 * k >= 1 with C_k >= p*C_N (p*C_N is one fp64 product), p >= 1 keeps N.  Each iteration evaluates
 * the midpoint and stops when |sum_l k_l - budget_tokens| <= tol_tokens, after max_iters
 * evaluations, or when the midpoint no longer differs from an end of the interval.
 *   budget_tokens <= L   -> all lengths 1, p = 0, iters = 0;
 *   budget_tokens >= L*N -> all lengths N, p = 1, iters = 0 (budget of 100%: no compression).
 * If fixup != 0 and the total missed the budget, the configuration is rescaled proportionally
 * (Sec. 3.3, last sentence of "Binary search for optimal configuration"): k_l*budget/total rounded
 * down and clamped to [1,N], then the remaining tokens are handed out one per layer in order of
 * largest remainder (ties: lower layer), cyclically, so that sum_l lengths == budget_tokens.
 *   lengths [B,L] i32, p_out [B] f64 (last evaluated midpoint), iters [B] i32 (evaluated
 *   midpoints), raw_total [B] i64 (sum of lengths before the rescale), status [B] i32
 *   (PKV_DEV_* bits; if non-zero the sequence gets lengths = 0, p = 0, iters = 0, raw_total = 0
 *   and its order/cum/prefix contents are unspecified).  All outputs [dev]. */
typedef struct {
    int64_t budget_tokens; /* per sequence */
    int64_t tol_tokens;    /* >= 0 */
    int32_t max_iters;     /* >= 1; 64 always reaches the stopping interval */
    int32_t fixup;         /* 0 / 1 */
} pkv_select_params;

/*   ws [dev]: prefixkv_workspace_bytes(PKV_OP_SELECT, shape, 0) bytes, 16-byte aligned (else
 *   PKV_ERR_WORKSPACE); contents on entry and after the call are unspecified.  It holds one status word per (sequence, layer) and, per layer, the prefix
 *   lengths at the 255 ratios t/256: the first eight bisection steps of Algorithm 1 can only ask for
 *   those, so the search serves them from that table (same lengths, same p, same iteration count as
 *   walking the cumulative sums) and reads the sums only from the ninth step on. */
int prefixkv_select(int B, int L, int N, const float *importance /* [dev] [B,L,N] */,
                    const pkv_select_params *params /* [host] */, int32_t *order, uint64_t *cum,
                    float *prefix, int32_t *lengths, double *p_out, int32_t *iters,
                    int64_t *raw_total, int32_t *status, void *ws, size_t ws_bytes,
                    pkv_stream stream);

/* ---- prefixkv_select for callers that cannot allocate device memory at all and therefore have no
 * workspace to pass: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, same kernels and bit-identical results as prefixkv_select, except that
 * the search takes every bisection step on the cumulative sums (no table of tabulated ratios, which
 * would need 1 KB per layer); the scratch
 * (one status word per (sequence, layer)) is a fixed array built into the library instead of `ws`:
 * 65536 words = 256 KB, which every GPU the library runs on holds until the process ends.
 *   B * L <= prefixkv_static_scratch_segments() (= 65536), else PKV_ERR_WORKSPACE, nothing enqueued.
 * The call allocates nothing and frees nothing.  The first call on a device looks up the array's
 * device address (with that device current) and keeps it for the life of the process.
 * All calls on one GPU share that GPU's array: two calls that may overlap in time on the same GPU
 * (different streams without an ordering event) race on it; calls on one stream are safe.  The
 * array's contents after a call are unspecified and nothing in it needs clearing between calls. */
int prefixkv_select_static(int B, int L, int N, const float *importance /* [dev] [B,L,N] */,
                           const pkv_select_params *params /* [host] */, int32_t *order,
                           uint64_t *cum, float *prefix, int32_t *lengths, double *p_out,
                           int32_t *iters, int64_t *raw_total, int32_t *status, pkv_stream stream);
int prefixkv_static_scratch_segments(void);

/* ---- Stage 2 alone, for offline estimation (Sec. 3.3, last paragraph: the retention ratios R_l
 * are estimated once from a few random samples and reused).  Same order / cum / prefix as
 * prefixkv_select and the same status bits, no search.  status [B] i32 = OR over the sequence's
 * layers; a sequence with a non-zero status has unspecified order/cum/prefix.  The workspace size
 * is that of PKV_OP_SELECT.  prefix may be NULL. */
int prefixkv_rank(int B, int L, int N, const float *importance /* [dev] [B,L,N] */, int32_t *order,
                  uint64_t *cum, float *prefix, int32_t *status, void *ws, size_t ws_bytes,
                  pkv_stream stream);

/* ---- Offline configuration (Sec. 3.3, last paragraph; Sec. 4.3 "offline estimation").
 * sample_lengths [dev] i32 [S,L]: the per-layer lengths prefixkv_select found for S calibration
 * sequences (each of them lengths/N = the sample's retention ratios R_l, same N for all samples).
 * The shared configuration is the mean of the samples' ratios, brought to the exact budget: with
 * weight_l = sum_s sample_lengths[s,l] and K = sum_l weight_l,
 *   lengths_l = weight_l*budget_tokens/K rounded down and clamped to [1,N], then the remaining
 *   tokens one per layer by largest remainder (ties: lower layer), cyclically, exactly as the
 *   rescale of prefixkv_select.  budget_tokens <= L -> all 1; >= L*N -> all N; K == 0 (every
 *   sample was rejected by its status word) -> all 0.
 * The paper fixes only "estimate offline from random samples"; the mean over samples is this
 * library's reading.  lengths_out [dev] i32 [B_out,L]: the same row B_out times, ready to be the
 * `lengths` of prefixkv_compact together with each sequence's own `order` from prefixkv_rank.
 * 1 <= S <= 65536, B_out >= 1.  No workspace. */
int prefixkv_offline_config(int S, int L, int N, const int32_t *sample_lengths,
                            int64_t budget_tokens, int B_out, int32_t *lengths_out,
                            pkv_stream stream);

/* ---- Stage 4a: compaction (Sec. 3.2: the top R_l proportion of KV vectors is retained in each
 * head of layer l; Fig. 3(a): layer-wise compressed cache).
 * The kept set of (b,l) is order[b,l,0..lengths[b,l]); it is stored in ascending position.
 * Ragged layout, computed on the device: caps[b,l] = lengths[b,l] + decode_capacity,
 * seg_off[b,l] = exclusive prefix sum of caps in (b,l) order (in tokens); segment (b,l) of kc/vc
 * is the [Hkv][caps][D] block starting at element seg_off*Hkv*D; kept_pos uses the same token
 * offsets (one int per slot).  lens[b,l] = lengths[b,l] = the number of occupied slots.
 * kc, vc must hold at least prefixkv_cache_tokens_upper_bound() tokens * Hkv * D elements and
 * kept_pos that many ints.  Slots beyond lens are not written.
 * N + decode_capacity must stay below 2^20 slots (PKV_ERR_DIM otherwise): the decode entry points
 * keep a completion count above bit 20 of lens and address a segment's rows with 32-bit offsets.
 *   k, v [dev] [B,L,Hkv,N,D] with strides; order [dev] [B,L,N]; lengths [dev] [B,L]
 *   seg_off [dev] i64 [B,L], caps [dev] i32 [B,L], lens [dev] i32 [B,L]: out */
int prefixkv_compact(const pkv_shape *shape, const void *k, pkv_strides ks, const void *v,
                     pkv_strides vs, const int32_t *order, const int32_t *lengths,
                     int decode_capacity, int64_t *seg_off, int32_t *caps, void *kc, void *vc,
                     int32_t *kept_pos, int32_t *lens, void *ws, size_t ws_bytes,
                     pkv_stream stream);

/* ---- Cache merging by positional distance (Sec. 4.3, "Eviction or merging": the pruned vector at
 * position m is matched to the retained position n with the largest metric c = -|m - n| and every
 * retained vector becomes the average of itself and the pruned vectors matched to it; the variant the
 * paper calls "Position".  The paper reports it as neutral to slightly harmful, so it is optional).
 * Runs in place on the output of prefixkv_compact, before the first decode step: slot j of segment
 * (b,l) holds position kept_pos[j]; a pruned position half way between two kept ones goes to the lower
 * (first maximum of the metric); keys and values of all KV heads are averaged alike, fp32 sums in
 * a fixed order, one rounding to the storage dtype.  Only the first lens[b,l] slots are written.
 *   k, v [dev]: the uncompressed tensors given to prefixkv_compact;  everything else as produced by it.
 * prefixkv_merge_feature is the variant with the cosine metric. */
int prefixkv_merge_position(const pkv_shape *shape, const void *k, pkv_strides ks, const void *v,
                            pkv_strides vs, const int64_t *seg_off, const int32_t *caps,
                            const int32_t *kept_pos, const int32_t *lens, void *kc, void *vc,
                            pkv_stream stream);

/* ---- Cache merging by feature similarity (Sec. 4.3, "Eviction or merging", the variant the paper calls
 * "Feature": matching metric c^{mn} = cosine of the pruned vector m and the retained vector n; every
 * retained vector becomes the average of itself and the pruned vectors whose largest metric it holds).
 * The paper spells the operation out for the keys of one head and treats values and the other heads
 * "the same"; the reading implemented is the literal one: each (kv head, tensor) pair is matched and
 * merged on its own -- keys by the cosine of keys, values by the cosine of values.
 * Runs in place on the output of prefixkv_compact, before the first decode step, like
 * prefixkv_merge_position.  bf16 storage only (PKV_ERR_UNSUPPORTED otherwise); N * row stride of k and
 * of v must be below 2^31 elements.
 *   Decision arithmetic: dot products of the bf16 vectors accumulated in fp32 on the matrix cores,
 *   times the fp32 reciprocal norm of the retained vector (the norm of the pruned vector is common to
 *   all its candidates and left out); a vector of norm zero has metric 0 with everything; among equal
 *   metrics the retained vector at the lowest position wins.  Sums of a group are taken in fp32 in a
 *   fixed order, one rounding to bf16.
 *   match [dev] i32 [2,B,L,Hkv,N] (out): plane 0 for keys, 1 for values; the slot a pruned position
 *       was merged into, -1 for a retained position.
 *   ws [dev]: prefixkv_workspace_bytes(PKV_OP_MERGE_FEATURE, shape, 0) bytes (the reciprocal norms). */
int prefixkv_merge_feature(const pkv_shape *shape, const void *k, pkv_strides ks, const void *v,
                           pkv_strides vs, const int64_t *seg_off, const int32_t *caps,
                           const int32_t *kept_pos, const int32_t *lens, void *kc, void *vc,
                           int32_t *match, void *ws, size_t ws_bytes, pkv_stream stream);

/* ---- Diagnostic: Gini coefficient of every layer's priority sequence (Sec. 4.3, "Relation between KV
 * cache size and importance distribution": layers with a more concentrated distribution, i.e. a higher
 * coefficient, receive smaller caches).  From the exact cumulative sums of prefixkv_select / _rank:
 *   gini[b,l] = (2 * (C_1 + ... + C_N) / C_N - N - 1) / N   (Lorenz curve, trapezoid rule);
 * 0 for a flat layer, (N-1)/N when one position holds everything, 0 when C_N = 0.
 *   cum [dev] u64 [B,L,N];  gini [dev] f64 [B,L]. */
int prefixkv_gini(int B, int L, int N, const uint64_t *cum, double *gini, pkv_stream stream);

/* Tokens to allocate for kc/vc/kept_pos when every sequence keeps at most `budget_tokens`. */
int64_t prefixkv_cache_tokens_upper_bound(int B, int64_t budget_tokens, int L, int decode_capacity);

/* ---- Stage 4b: one decode step over layers [l0,l1) (Sec. 3.1: the newest token's query
 * interacts with the cached KV vectors).  One kernel launch.
 * If k_new/v_new are non-NULL, the new token's key/value of every (b,l,kv head) are first stored
 * in slot lens[b,l] of the segment and lens[b,l] becomes lens[b,l]+1 (the caller guarantees
 * lens < caps; a full segment drops the append and the step attends over the old slots).  Then
 *   out[b,l,h,:] = sum_j softmax_j(scale[l] * q[b,l,h,:].kc_j) * vc_j   over the lens slots of kv
 * head g(h); an empty segment gives zeros.  fp32 softmax and accumulation; out in shape->dtype.
 *   q, out [dev] [B,L,H,D] dense;  k_new, v_new [dev] [B,L,Hkv,D] dense or NULL (both)
 *   kc, vc, seg_off, caps as produced by prefixkv_compact (every caps entry below 2^20, which
 *       prefixkv_compact enforces through N + decode_capacity < 2^20)
 *   lens [dev] in/out: plain lengths below 2^20 before and after the call.  WHILE the launch runs
 *       the library keeps a completion count in the bits above 2^20 of each entry, so lens must
 *       not be read or written by anything else until the launch has finished.  H <= 2048.
 *   ws: needed when several query heads share a KV head and the cache is bf16 (the segments are cut into
 *       pieces of similar size and the pieces' partial results meet in the workspace);
 *       prefixkv_workspace_bytes(PKV_OP_DECODE, shape, 0) gives the size (0 when none is needed, then
 *       ws may be NULL).  The size is for layer range [0,L); a smaller workspace is PKV_ERR_WORKSPACE. */
int prefixkv_decode_attn(const pkv_shape *shape, int l0, int l1, const void *q, const void *k_new,
                         const void *v_new, const float *scale, void *kc, void *vc,
                         const int64_t *seg_off, const int32_t *caps, int32_t *lens, void *out,
                         void *ws, size_t ws_bytes, pkv_stream stream);

/* ---- Decode step with ratio maintenance (Sec. 3.1, last sentences, and the caption of Fig. 3:
 * while decoding, the vectors at a fixed distance to the latest generated token are pruned so that
 * the prefix configuration found after prefill keeps holding).  The paper states neither the
 * distance nor the bookkeeping; this library's reading:
 *   R_l = base_lens[b,l] / N;  after decode step t (1-based; the sequence then has N+t tokens) the
 *   segment aims at  target(t) = max(1, floor((2*base_lens*(N+t) + N) / (2N)))  entries
 *   (= R_l*(N+t) rounded half up).  Step t stores the new token, then decides the token stored
 *   `distance` steps earlier, once: it becomes a permanent entry if the cache including it is within
 *   target(t), else it is dropped.  Steps t <= distance decide nothing.  The `distance` newest tokens
 *   are always cached.  The query of step t attends to the cache AFTER this decision.  The number of
 *   cached entries after step t is max(target(t), base_lens + min(t, distance)).
 * Segment layout: slots [0, lens) are permanent entries (the kept prompt positions from
 * prefixkv_compact, then survivors in the order they were decided); the LAST distance+1 slots of
 * the segment (caps - distance - 1 ... caps - 1) are a ring, decode token j in ring slot
 * (j-1) mod (distance+1).  lens[b,l] counts PERMANENT entries only and must come from
 * prefixkv_compact (t = 1) or the previous call (t-1) with the same distance; a cache driven through
 * this entry point must not be passed to prefixkv_decode_attn.  prefixkv_compact must have been
 * called with decode_capacity >= distance+1 + the number of survivors the caller will allow
 * (never more than the number of steps).  A segment whose capacity cannot hold the ring behind its
 * kept prompt entries is left untouched and outputs zeros; a survivor that does not fit in front of
 * the ring is dropped.
 *   base_lens [dev] i32 [B,L]: the `lengths` given to prefixkv_compact (read only)
 *   kept_pos  [dev] i32 or NULL: if given, slot labels are maintained: N+j-1 for decode token j in the
 *       ring and in the permanent region, -1 for a ring slot whose token was decided
 *   t: 1-based decode step since prefixkv_compact;  1 <= distance <= 65535
 * Everything else as in prefixkv_decode_attn (k_new, v_new required; caps below 2^20). */
int prefixkv_decode_attn_evict(const pkv_shape *shape, int l0, int l1, const void *q,
                               const void *k_new, const void *v_new, const float *scale, void *kc,
                               void *vc, const int64_t *seg_off, const int32_t *caps,
                               const int32_t *base_lens, int32_t *lens, int32_t *kept_pos, int t,
                               int distance, void *out, void *ws, size_t ws_bytes,
                               pkv_stream stream);

/* Measurement aid, not part of the method: a plain device-to-device copy kernel of a known size
 * (bytes % 16 == 0, 16-byte aligned pointers).  It reads `bytes` and writes `bytes`, which is what
 * hardware byte counters are calibrated against when a kernel's HBM traffic is reported. */
int prefixkv_calibration_copy(void *dst /* [dev] */, const void *src /* [dev] */, size_t bytes,
                              pkv_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* PREFIXKV_H */
