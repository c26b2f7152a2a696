// Shared declarations of the HIP side of libprefixkv: launcher prototypes (one per stage, defined
// next to their kernels) and a few device helpers.  gfx950 only, wave64.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/prefixkv.h"

namespace pkv {

constexpr int kWave = 64;
constexpr int kMaxL = 64;
constexpr int kMaxN = 8192;
constexpr int64_t kMaxSegmentSlots = 1 << 20;   // slots of one (b,l) segment: prompt entries + decode capacity
constexpr int kDecodeChunk = 64;   // tokens of one (b,l,kv-head) segment handled by one wave
constexpr int kXcds = 8;           // L2 slices (XCDs) of the chip; workgroup id % 8 picks the XCD

typedef unsigned short bf16_t;     // raw bfloat16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t x) { return __uint_as_float(((uint32_t)x) << 16); }
// round to nearest even; NaN stays NaN
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

// Consecutive workgroup ids land on different XCDs; map them so that `nblk/8` consecutive logical
// ids share an XCD (and its L2).  nblk must be a multiple of 8.
__device__ __forceinline__ uint32_t xcd_swizzle(uint32_t bid, uint32_t nblk) {
    return (bid % kXcds) * (nblk / kXcds) + bid / kXcds;
}

struct Strides { int64_t b, l, h, n; };
inline Strides to_strides(pkv_strides s) { return Strides{s.b, s.l, s.h, s.n}; }

// ---- launchers (return hipError_t of the launches) -------------------------------------------------
size_t importance_ws_bytes(const pkv_shape& s, bool has_lse);
hipError_t launch_importance(const pkv_shape& s, const void* q, Strides qs, const void* k, Strides ks,
                             const float* scale, const float* lse, float* importance, void* ws,
                             hipStream_t st);

hipError_t launch_prefill_attn(const pkv_shape& s, const void* q, Strides qs, const void* k, Strides ks,
                               const void* v, Strides vs, const float* scale, void* out, float* lse,
                               hipStream_t st);

size_t select_ws_bytes(int B, int L, int N);
hipError_t launch_select(int B, int L, int N, const float* importance, const pkv_select_params& p,
                         int32_t* order, uint64_t* cum, float* prefix, int32_t* lengths, double* p_out,
                         int32_t* iters, int64_t* raw_total, int32_t* status, void* ws, bool with_table,
                         hipStream_t st);

int select_static_max_segments();
hipError_t launch_select_static(int B, int L, int N, const float* importance, const pkv_select_params& p,
                                int32_t* order, uint64_t* cum, float* prefix, int32_t* lengths, double* p_out,
                                int32_t* iters, int64_t* raw_total, int32_t* status, hipStream_t st);

hipError_t launch_rank(int B, int L, int N, const float* importance, int32_t* order, uint64_t* cum,
                       float* prefix, int32_t* status, void* ws, hipStream_t st);
hipError_t launch_offline_config(int S, int L, int N, const int32_t* sample_lengths, int64_t budget,
                                 int copies, int32_t* lengths, hipStream_t st);

hipError_t launch_gini(int B, int L, int N, const uint64_t* cum, double* gini, hipStream_t st);
hipError_t launch_merge_position(const pkv_shape& s, const void* k, Strides ks, const void* v, Strides vs,
                                 const int64_t* seg_off, const int32_t* caps, const int32_t* kept_pos,
                                 const int32_t* lens, void* kc, void* vc, hipStream_t st);

size_t merge_feature_ws_bytes(const pkv_shape& s);
hipError_t launch_merge_feature(const pkv_shape& s, const void* k, Strides ks, const void* v, Strides vs,
                                const int64_t* seg_off, const int32_t* caps, const int32_t* kept_pos,
                                const int32_t* lens, void* kc, void* vc, int32_t* match, void* ws,
                                hipStream_t st);

size_t compact_ws_bytes(const pkv_shape& s);
hipError_t launch_compact(const pkv_shape& s, const void* k, Strides ks, const void* v, Strides vs,
                          const int32_t* order, const int32_t* lengths, int decode_capacity,
                          int64_t* seg_off, int32_t* caps, void* kc, void* vc, int32_t* kept_pos,
                          int32_t* lens, void* ws, hipStream_t st);

size_t decode_ws_bytes(const pkv_shape& s);
hipError_t launch_decode(const pkv_shape& s, int l0, int l1, const void* q, const void* k_new,
                         const void* v_new, const float* scale, void* kc, void* vc,
                         const int64_t* seg_off, const int32_t* caps, int32_t* lens, void* out, void* ws,
                         hipStream_t st);
hipError_t launch_decode_evict(const pkv_shape& s, int l0, int l1, const void* q, const void* k_new,
                               const void* v_new, const float* scale, void* kc, void* vc,
                               const int64_t* seg_off, const int32_t* caps, const int32_t* base_lens,
                               int32_t* lens, int32_t* kept_pos, int t, int d, void* out, void* ws,
                               hipStream_t st);

}  // namespace pkv
