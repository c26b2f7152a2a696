// C ABI of libprefixkv: argument validation and dispatch.  No allocation, no synchronisation; every
// launch goes to the caller's stream.  The only state kept between calls is looked up once per device:
// the compute-unit count, and the address of the built-in scratch array of prefixkv_select_static.
#include "pkv_common.hpp"

using namespace pkv;

namespace {

// Plain copy, 16 bytes per lane, grid-stride: the known-size reference for calibrating byte counters.
__global__ void __launch_bounds__(256) calibration_copy_kernel(const uint4* __restrict__ src,
                                                               uint4* __restrict__ dst, size_t n16) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

bool shape_ok(const pkv_shape* s) {
    return s->B >= 1 && s->L >= 1 && s->L <= kMaxL && s->H >= 1 && s->Hkv >= 1 && s->H % s->Hkv == 0 &&
           s->N >= 1 && s->N <= kMaxN && (s->D == 64 || s->D == 128);
}
bool dtype_ok(const pkv_shape* s) { return s->dtype == PKV_F32 || s->dtype == PKV_BF16; }
// rows are moved in 16-byte pieces
bool strides_ok(const pkv_strides& t, int esize) {
    const int64_t a = 16 / esize;
    return t.b >= 0 && t.l >= 0 && t.h >= 0 && t.n > 0 && t.b % a == 0 && t.l % a == 0 && t.h % a == 0 &&
           t.n % a == 0;
}
bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

}  // namespace

extern "C" {

int prefixkv_version(void) { return 100; }

const char* prefixkv_status_string(int status) {
    switch (status) {
        case PKV_OK: return "ok";
        case PKV_ERR_NULL: return "required pointer is NULL";
        case PKV_ERR_DIM: return "dimension out of range";
        case PKV_ERR_DTYPE: return "unknown dtype";
        case PKV_ERR_STRIDE: return "stride or pointer not 16-byte aligned";
        case PKV_ERR_WORKSPACE: return "workspace missing or too small";
        case PKV_ERR_BUDGET: return "invalid budget, tolerance or iteration limit";
        case PKV_ERR_UNSUPPORTED: return "unsupported configuration";
        case PKV_ERR_HIP: return "kernel launch failed";
        default: return "unknown status";
    }
}

size_t prefixkv_workspace_bytes(int op, const pkv_shape* s, int has_lse) {
    if (!s || !shape_ok(s) || !dtype_ok(s)) return 0;
    switch (op) {
        case PKV_OP_IMPORTANCE: return importance_ws_bytes(*s, has_lse != 0);
        case PKV_OP_SELECT: return select_ws_bytes(s->B, s->L, s->N);
        case PKV_OP_COMPACT: return compact_ws_bytes(*s);
        case PKV_OP_DECODE: return decode_ws_bytes(*s);
        case PKV_OP_MERGE_FEATURE: return merge_feature_ws_bytes(*s);
        default: return 0;
    }
}

int prefixkv_importance(const pkv_shape* s, const void* q, pkv_strides qs, const void* k, pkv_strides ks,
                        const float* scale, const float* lse, float* importance, void* ws,
                        size_t ws_bytes, pkv_stream stream) {
    if (!s || !q || !k || !scale || !importance) return PKV_ERR_NULL;
    if (!shape_ok(s)) return PKV_ERR_DIM;
    if (!dtype_ok(s)) return PKV_ERR_DTYPE;
    const int esize = s->dtype == PKV_F32 ? 4 : 2;
    if (!strides_ok(qs, esize) || !strides_ok(ks, esize) || !aligned16(q) || !aligned16(k))
        return PKV_ERR_STRIDE;
    // the bf16 kernels address the rows of one head with 32-bit element offsets
    if ((uint64_t)s->N * (uint64_t)qs.n >= (1ull << 31) || (uint64_t)s->N * (uint64_t)ks.n >= (1ull << 31))
        return PKV_ERR_UNSUPPORTED;
    if (!ws || ws_bytes < importance_ws_bytes(*s, lse != nullptr)) return PKV_ERR_WORKSPACE;
    const hipError_t e = launch_importance(*s, q, to_strides(qs), k, to_strides(ks), scale, lse, importance,
                                           ws, (hipStream_t)stream);
    return e == hipSuccess ? PKV_OK : PKV_ERR_HIP;
}

int prefixkv_prefill_attn(const pkv_shape* s, const void* q, pkv_strides qs, const void* k, pkv_strides ks,
                          const void* v, pkv_strides vs, const float* scale, void* out, float* lse,
                          pkv_stream stream) {
    if (!s || !q || !k || !v || !scale || !out || !lse) return PKV_ERR_NULL;
    if (!shape_ok(s)) return PKV_ERR_DIM;
    if (!dtype_ok(s)) return PKV_ERR_DTYPE;
    if (s->dtype != PKV_BF16) return PKV_ERR_UNSUPPORTED;
    if (!strides_ok(qs, 2) || !strides_ok(ks, 2) || !strides_ok(vs, 2) || !aligned16(q) || !aligned16(k) ||
        !aligned16(v) || !aligned16(out))
        return PKV_ERR_STRIDE;
    if ((size_t)s->B * s->L * s->H * ((s->N + 127) / 128) > 0x7fffffffull) return PKV_ERR_UNSUPPORTED;
    if ((uint64_t)s->N * (uint64_t)ks.n >= (1ull << 31) || (uint64_t)s->N * (uint64_t)vs.n >= (1ull << 31))
        return PKV_ERR_UNSUPPORTED;   // rows of one head are addressed with 32-bit element offsets
    const hipError_t e = launch_prefill_attn(*s, q, to_strides(qs), k, to_strides(ks), v, to_strides(vs), scale, out,
                                             lse, (hipStream_t)stream);
    return e == hipSuccess ? PKV_OK : PKV_ERR_HIP;
}

int prefixkv_select(int B, int L, int N, const float* importance, const pkv_select_params* params,
                    int32_t* order, uint64_t* cum, float* prefix, int32_t* lengths, double* p_out,
                    int32_t* iters, int64_t* raw_total, int32_t* status, void* ws, size_t ws_bytes,
                    pkv_stream stream) {
    if (!importance || !params || !order || !cum || !lengths || !p_out || !iters || !raw_total || !status)
        return PKV_ERR_NULL;
    if (B < 1 || L < 1 || L > kMaxL || N < 1 || N > kMaxN) return PKV_ERR_DIM;
    if (params->budget_tokens < 1 || params->tol_tokens < 0 || params->max_iters < 1) return PKV_ERR_BUDGET;
    if (!ws || ws_bytes < select_ws_bytes(B, L, N) || !aligned16(ws)) return PKV_ERR_WORKSPACE;
    const hipError_t e = launch_select(B, L, N, importance, *params, order, cum, prefix, lengths, p_out,
                                       iters, raw_total, status, ws, true, (hipStream_t)stream);
    return e == hipSuccess ? PKV_OK : PKV_ERR_HIP;
}

int prefixkv_select_static(int B, int L, int N, const float* importance, const pkv_select_params* params,
                           int32_t* order, uint64_t* cum, float* prefix, int32_t* lengths, double* p_out,
                           int32_t* iters, int64_t* raw_total, int32_t* status, pkv_stream stream) {
    if (!importance || !params || !order || !cum || !lengths || !p_out || !iters || !raw_total || !status)
        return PKV_ERR_NULL;
    if (B < 1 || L < 1 || L > kMaxL || N < 1 || N > kMaxN) return PKV_ERR_DIM;
    if (params->budget_tokens < 1 || params->tol_tokens < 0 || params->max_iters < 1) return PKV_ERR_BUDGET;
    // the built-in scratch array holds one word per (sequence, layer)
    if ((int64_t)B * L > select_static_max_segments()) return PKV_ERR_WORKSPACE;
    const hipError_t e = launch_select_static(B, L, N, importance, *params, order, cum, prefix, lengths, p_out,
                                              iters, raw_total, status, (hipStream_t)stream);
    return e == hipSuccess ? PKV_OK : PKV_ERR_HIP;
}

int prefixkv_static_scratch_segments(void) { return select_static_max_segments(); }

int prefixkv_rank(int B, int L, int N, const float* importance, int32_t* order, uint64_t* cum, float* prefix,
                  int32_t* status, void* ws, size_t ws_bytes, pkv_stream stream) {
    if (!importance || !order || !cum || !status) return PKV_ERR_NULL;
    if (B < 1 || L < 1 || L > kMaxL || N < 1 || N > kMaxN) return PKV_ERR_DIM;
    if (!ws || ws_bytes < select_ws_bytes(B, L, N)) return PKV_ERR_WORKSPACE;
    const hipError_t e = launch_rank(B, L, N, importance, order, cum, prefix, status, ws, (hipStream_t)stream);
    return e == hipSuccess ? PKV_OK : PKV_ERR_HIP;
}

int prefixkv_offline_config(int S, int L, int N, const int32_t* sample_lengths, int64_t budget_tokens,
                            int B_out, int32_t* lengths_out, pkv_stream stream) {
    if (!sample_lengths || !lengths_out) return PKV_ERR_NULL;
    if (S < 1 || S > 65536 || L < 1 || L > kMaxL || N < 1 || N > kMaxN || B_out < 1) return PKV_ERR_DIM;
    if (budget_tokens < 1) return PKV_ERR_BUDGET;
    const hipError_t e = launch_offline_config(S, L, N, sample_lengths, budget_tokens, B_out, lengths_out,
                                               (hipStream_t)stream);
    return e == hipSuccess ? PKV_OK : PKV_ERR_HIP;
}

int prefixkv_compact(const pkv_shape* s, const void* k, pkv_strides ks, const void* v, pkv_strides vs,
                     const int32_t* order, const int32_t* lengths, int decode_capacity, int64_t* seg_off,
                     int32_t* caps, void* kc, void* vc, int32_t* kept_pos, int32_t* lens, void* ws,
                     size_t ws_bytes, pkv_stream stream) {
    if (!s || !k || !v || !order || !lengths || !seg_off || !caps || !kc || !vc || !kept_pos || !lens)
        return PKV_ERR_NULL;
    if (!shape_ok(s) || decode_capacity < 0) return PKV_ERR_DIM;
    // the decode kernels keep a completion count in bits 20 and up of lens and address the rows of a
    // segment with 32-bit byte offsets: a segment (N + decode_capacity slots at most) stays below 2^20
    if ((int64_t)s->N + decode_capacity >= kMaxSegmentSlots) return PKV_ERR_DIM;
    if (!dtype_ok(s)) return PKV_ERR_DTYPE;
    const int esize = s->dtype == PKV_F32 ? 4 : 2;
    if (!strides_ok(ks, esize) || !strides_ok(vs, esize) || !aligned16(k) || !aligned16(v) ||
        !aligned16(kc) || !aligned16(vc))
        return PKV_ERR_STRIDE;
    if ((size_t)((s->N + 63) / 64) * s->Hkv * s->B * s->L > 0x7fffffffull) return PKV_ERR_UNSUPPORTED;
    (void)ws; (void)ws_bytes;  // this stage needs no scratch
    const hipError_t e = launch_compact(*s, k, to_strides(ks), v, to_strides(vs), order, lengths,
                                        decode_capacity, seg_off, caps, kc, vc, kept_pos, lens, ws,
                                        (hipStream_t)stream);
    return e == hipSuccess ? PKV_OK : PKV_ERR_HIP;
}

int prefixkv_gini(int B, int L, int N, const uint64_t* cum, double* gini, pkv_stream stream) {
    if (!cum || !gini) return PKV_ERR_NULL;
    if (B < 1 || L < 1 || L > kMaxL || N < 1 || N > kMaxN) return PKV_ERR_DIM;
    const hipError_t e = launch_gini(B, L, N, cum, gini, (hipStream_t)stream);
    return e == hipSuccess ? PKV_OK : PKV_ERR_HIP;
}

int prefixkv_merge_position(const pkv_shape* s, const void* k, pkv_strides ks, const void* v, pkv_strides vs,
                            const int64_t* seg_off, const int32_t* caps, const int32_t* kept_pos,
                            const int32_t* lens, void* kc, void* vc, pkv_stream stream) {
    if (!s || !k || !v || !seg_off || !caps || !kept_pos || !lens || !kc || !vc) return PKV_ERR_NULL;
    if (!shape_ok(s)) return PKV_ERR_DIM;
    if (!dtype_ok(s)) return PKV_ERR_DTYPE;
    const int esize = s->dtype == PKV_F32 ? 4 : 2;
    if (!strides_ok(ks, esize) || !strides_ok(vs, esize) || !aligned16(k) || !aligned16(v) ||
        !aligned16(kc) || !aligned16(vc))
        return PKV_ERR_STRIDE;
    if ((size_t)8 * s->Hkv * s->B * s->L > 0x7fffffffull) return PKV_ERR_UNSUPPORTED;
    const hipError_t e = launch_merge_position(*s, k, to_strides(ks), v, to_strides(vs), seg_off, caps, kept_pos,
                                               lens, kc, vc, (hipStream_t)stream);
    return e == hipSuccess ? PKV_OK : PKV_ERR_HIP;
}

int prefixkv_merge_feature(const pkv_shape* s, const void* k, pkv_strides ks, const void* v, pkv_strides vs,
                           const int64_t* seg_off, const int32_t* caps, const int32_t* kept_pos,
                           const int32_t* lens, void* kc, void* vc, int32_t* match, void* ws, size_t ws_bytes,
                           pkv_stream stream) {
    if (!s || !k || !v || !seg_off || !caps || !kept_pos || !lens || !kc || !vc || !match) return PKV_ERR_NULL;
    if (!shape_ok(s)) return PKV_ERR_DIM;
    if (!dtype_ok(s)) return PKV_ERR_DTYPE;
    if (s->dtype != PKV_BF16) return PKV_ERR_UNSUPPORTED;
    if (!strides_ok(ks, 2) || !strides_ok(vs, 2) || !aligned16(k) || !aligned16(v) || !aligned16(kc) ||
        !aligned16(vc))
        return PKV_ERR_STRIDE;
    // the kernels address rows with 32-bit element offsets, and their grids are one-dimensional
    if ((int64_t)s->N * ks.n > 0x7fffffffll || (int64_t)s->N * vs.n > 0x7fffffffll ||
        (size_t)2 * 64 * s->Hkv * s->B * s->L > 0x7fffffffull)
        return PKV_ERR_UNSUPPORTED;
    if (!ws || ws_bytes < merge_feature_ws_bytes(*s) || !aligned16(ws)) return PKV_ERR_WORKSPACE;
    const hipError_t e = launch_merge_feature(*s, k, to_strides(ks), v, to_strides(vs), seg_off, caps, kept_pos,
                                              lens, kc, vc, match, ws, (hipStream_t)stream);
    return e == hipSuccess ? PKV_OK : PKV_ERR_HIP;
}

int64_t prefixkv_cache_tokens_upper_bound(int B, int64_t budget_tokens, int L, int decode_capacity) {
    if (B < 1 || L < 1 || budget_tokens < 0 || decode_capacity < 0) return 0;
    return (int64_t)B * (budget_tokens + (int64_t)L * decode_capacity);
}

int prefixkv_decode_attn(const pkv_shape* s, int l0, int l1, const void* q, const void* k_new,
                         const void* v_new, const float* scale, void* kc, void* vc, const int64_t* seg_off,
                         const int32_t* caps, int32_t* lens, void* out, void* ws, size_t ws_bytes,
                         pkv_stream stream) {
    if (!s || !q || !scale || !kc || !vc || !seg_off || !caps || !lens || !out) return PKV_ERR_NULL;
    if ((k_new == nullptr) != (v_new == nullptr)) return PKV_ERR_NULL;
    if (!shape_ok(s) || l0 < 0 || l1 > s->L || l0 >= l1 || s->H > 2048) return PKV_ERR_DIM;
    if (!dtype_ok(s)) return PKV_ERR_DTYPE;
    if (!aligned16(q) || !aligned16(kc) || !aligned16(vc) || !aligned16(out) || !aligned16(k_new) ||
        !aligned16(v_new))
        return PKV_ERR_STRIDE;
    const size_t need = decode_ws_bytes(*s);
    if (need > 0 && (ws == nullptr || ws_bytes < need)) return PKV_ERR_WORKSPACE;
    const hipError_t e = launch_decode(*s, l0, l1, q, k_new, v_new, scale, kc, vc, seg_off, caps, lens, out, ws,
                                       (hipStream_t)stream);
    return e == hipSuccess ? PKV_OK : PKV_ERR_HIP;
}

int prefixkv_decode_attn_evict(const pkv_shape* s, int l0, int l1, const void* q, const void* k_new,
                               const void* v_new, const float* scale, void* kc, void* vc,
                               const int64_t* seg_off, const int32_t* caps, const int32_t* base_lens,
                               int32_t* lens, int32_t* kept_pos, int t, int distance, void* out, void* ws,
                               size_t ws_bytes, pkv_stream stream) {
    if (!s || !q || !k_new || !v_new || !scale || !kc || !vc || !seg_off || !caps || !base_lens || !lens || !out)
        return PKV_ERR_NULL;
    if (!shape_ok(s) || l0 < 0 || l1 > s->L || l0 >= l1 || s->H > 2048) return PKV_ERR_DIM;
    if (t < 1 || t > (1 << 30) || distance < 1 || distance > 65535) return PKV_ERR_DIM;
    if (!dtype_ok(s)) return PKV_ERR_DTYPE;
    if (!aligned16(q) || !aligned16(kc) || !aligned16(vc) || !aligned16(out) || !aligned16(k_new) ||
        !aligned16(v_new))
        return PKV_ERR_STRIDE;
    const size_t need = decode_ws_bytes(*s);
    if (need > 0 && (ws == nullptr || ws_bytes < need)) return PKV_ERR_WORKSPACE;
    const hipError_t e = launch_decode_evict(*s, l0, l1, q, k_new, v_new, scale, kc, vc, seg_off, caps, base_lens,
                                             lens, kept_pos, t, distance, out, ws, (hipStream_t)stream);
    return e == hipSuccess ? PKV_OK : PKV_ERR_HIP;
}

int prefixkv_calibration_copy(void* dst, const void* src, size_t bytes, pkv_stream stream) {
    if (!dst || !src) return PKV_ERR_NULL;
    if (bytes == 0 || bytes % 16 != 0) return PKV_ERR_DIM;
    if (!aligned16(dst) || !aligned16(src)) return PKV_ERR_STRIDE;
    hipLaunchKernelGGL(calibration_copy_kernel, dim3(8192), dim3(256), 0, (hipStream_t)stream,
                       (const uint4*)src, (uint4*)dst, bytes / 16);
    return hipGetLastError() == hipSuccess ? PKV_OK : PKV_ERR_HIP;
}

}  // extern "C"
