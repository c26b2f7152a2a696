// Stage 4a: gather the kept K/V rows of every layer into the ragged per-layer cache (Sec. 3.2: the
// top R_l proportion is retained in each head of layer l; all heads of a layer share one index set).
//
//  compact_fused_kernel   one launch: every workgroup of a (sequence, layer, kv head, 64-row chunk) derives the
//                         segment's offset and its kept positions in ascending order (flag array in LDS ->
//                         exclusive scan -> scatter) and streams its whole rows (16 B per lane) from K/V into
//                         the segment.  Pure HBM traffic.
//  merge_position_kernel  the positional-distance merge of Sec. 4.3 on top of a compacted cache.
#include "pkv_common.hpp"

namespace pkv {

// Source rows are read once.  Loads that bypass the caches (nontemporal) pay when K and V together are far
// larger than the 256 MB last-level cache (from 2 GiB on, inside the whole pipeline: -5 % ... -7 %; below that
// they cost up to 20 %), so the launcher chooses.  Nontemporal stores of the cache rows were 2-5 % slower inside
// the pipeline at every size (and faster only when the same call is repeated back to back), so stores are plain.
typedef __attribute__((ext_vector_type(4))) unsigned int cu32x4_t;
template <bool NT>
__device__ __forceinline__ uint4 ld_row16(const unsigned char* p) {
    if constexpr (NT) {
        const cu32x4_t t = __builtin_nontemporal_load((const cu32x4_t*)p);
        return make_uint4(t.x, t.y, t.z, t.w);
    } else {
        return *(const uint4*)p;
    }
}

// One launch.  Every workgroup of a (segment, kv head, chunk) builds the segment's list of kept positions
// itself in LDS (flag per position -> counts -> exclusive scan -> scatter: ascending positions) and then copies
// its chunks of 64 rows, K and V, 16 bytes per lane (LPR lanes cover a row, so the workgroup moves 256/LPR
// whole rows per instruction); the workgroup of kv head 0, chunk 0 also writes the segment's offset (sum of the
// lengths and capacities of the segments before it), capacity, length and positions for the later stages.
// The redundant plans read `order` (4 bytes per kept row) from the L2 and cost less than the separate planning
// launch they replace (7B shape, batch 1: 35 -> 31 us; N = 8192: 171 -> 163 us).  Workgroups whose chunk lies
// beyond the segment's length leave at once; beyond 16 chunks a workgroup walks further chunks.
template <int LPR, bool NTL>
__global__ void __launch_bounds__(256)
compact_fused_kernel(int N, int nchunk, int Hkv, int L, int row_bytes, const unsigned char* __restrict__ k, Strides ks,
                     const unsigned char* __restrict__ v, Strides vs, int esize, const int32_t* __restrict__ order,
                     const int32_t* __restrict__ lengths, int decode_capacity, int64_t* __restrict__ seg_off,
                     int32_t* __restrict__ caps, int32_t* __restrict__ lens, int32_t* __restrict__ kept_pos,
                     unsigned char* __restrict__ kc, unsigned char* __restrict__ vc) {
    constexpr int kRows = 64;
    constexpr int RPI = 256 / LPR;
    extern __shared__ int s_dyn[];                  // kept positions (N ints), then the flags (N rounded up to 4 bytes)
    __shared__ int s_wave[4];
    __shared__ long long s_off[4];
    int* s_kept = s_dyn;
    uint32_t* s_flag = (uint32_t*)(s_dyn + N);
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    // chunk index fastest: neighbouring workgroups read neighbouring source rows and write adjacent slots.
    // `nchunk` is odd (see the launcher), so the chunks of successive (segment, head) pairs rotate over the XCDs.
    const int chunk = blockIdx.x % nchunk, h = (blockIdx.x / nchunk) % Hkv, seg = blockIdx.x / (nchunk * Hkv);
    int klen = lengths[seg];
    klen = klen < 0 ? 0 : (klen > N ? N : klen);
    const bool scribe = h == 0 && chunk == 0;
    if (chunk * kRows >= klen && !scribe) return;

    // token offset of the segment = sum of (length + capacity) of all segments before it
    long long acc = 0;
    for (int i = tid; i < seg; i += 256) acc += (long long)lengths[i] + decode_capacity;
    const int32_t* ord = order + (size_t)seg * N;
    int pos_mine[4];                                 // the first 1024 entries of the list are requested at once
#pragma unroll
    for (int u = 0; u < 4; ++u) pos_mine[u] = tid + 256 * u < klen ? ord[tid + 256 * u] : -1;
    const int nword = (N + 3) / 4;
    for (int i = tid; i < nword; i += 256) s_flag[i] = 0;
    for (int d = 32; d > 0; d >>= 1) {
        const uint32_t lo = __shfl_xor((uint32_t)acc, d, kWave);
        const uint32_t hi = __shfl_xor((uint32_t)((unsigned long long)acc >> 32), d, kWave);
        acc += (long long)(((unsigned long long)hi << 32) | lo);
    }
    if (lane == 0) s_off[wv] = acc;
    __syncthreads();
    const long long off = s_off[0] + s_off[1] + s_off[2] + s_off[3];
    unsigned char* fb = (unsigned char*)s_flag;
#pragma unroll
    for (int u = 0; u < 4; ++u)
        if (pos_mine[u] >= 0 && pos_mine[u] < N) fb[pos_mine[u]] = 1;
    for (int j = tid + 1024; j < klen; j += 256) {
        const int pos = ord[j];
        if (pos >= 0 && pos < N) fb[pos] = 1;
    }
    __syncthreads();
    // a thread owns E consecutive flag words
    const int E = (nword + 255) / 256;
    const int w_lo = tid * E, w_hi = min(w_lo + E, nword);
    int cnt = 0;
    for (int w = w_lo; w < w_hi; ++w) cnt += (int)((s_flag[w] * 0x01010101u) >> 24);
    int incl = cnt;
    for (int d = 1; d < kWave; d <<= 1) {
        const int up = __shfl_up(incl, d, kWave);
        if (lane >= d) incl += up;
    }
    if (lane == kWave - 1) s_wave[wv] = incl;
    __syncthreads();
    int at = incl - cnt;
    for (int w = 0; w < wv; ++w) at += s_wave[w];
    const int len = s_wave[0] + s_wave[1] + s_wave[2] + s_wave[3];   // = klen when `order` is a permutation
    for (int w = w_lo; w < w_hi; ++w) {
        const uint32_t f = s_flag[w];
#pragma unroll
        for (int x = 0; x < 4; ++x)
            if ((f >> (8 * x)) & 1) s_kept[at++] = 4 * w + x;
    }
    __syncthreads();
    if (scribe) {
        for (int j = tid; j < len; j += 256) kept_pos[off + j] = s_kept[j];
        if (tid == 0) {
            seg_off[seg] = off;
            caps[seg] = klen + decode_capacity;
            lens[seg] = klen;
        }
    }
    const int b = seg / L, l = seg % L;
    const int cap = klen + decode_capacity;
    const int sub = tid % LPR, rsel = tid / LPR;
    const unsigned char* kb = k + (ks.b * b + ks.l * l + ks.h * h) * (int64_t)esize;
    const unsigned char* vb = v + (vs.b * b + vs.l * l + vs.h * h) * (int64_t)esize;
    const int64_t dst0 = ((int64_t)off * Hkv + (int64_t)h * cap) * row_bytes;
    for (int r0 = chunk * kRows; r0 < len; r0 += nchunk * kRows) {
        uint4 kr[kRows / RPI], vr[kRows / RPI];
#pragma unroll
        for (int i = 0; i < kRows / RPI; ++i) {
            const int r = r0 + i * RPI + rsel;
            kr[i] = vr[i] = make_uint4(0, 0, 0, 0);
            if (r < len) {
                const int pos = s_kept[r];
                kr[i] = ld_row16<NTL>(kb + ks.n * pos * (int64_t)esize + sub * 16);
                vr[i] = ld_row16<NTL>(vb + vs.n * pos * (int64_t)esize + sub * 16);
            }
        }
#pragma unroll
        for (int i = 0; i < kRows / RPI; ++i) {
            const int r = r0 + i * RPI + rsel;
            if (r < len) {
                *(uint4*)(kc + dst0 + (int64_t)r * row_bytes + sub * 16) = kr[i];
                *(uint4*)(vc + dst0 + (int64_t)r * row_bytes + sub * 16) = vr[i];
            }
        }
    }
}

// Cache merging by positional distance (Sec. 4.3, "Eviction or merging", metric -|m - n|): every pruned
// position is averaged into the nearest kept one (half way: the lower), keys and values of all heads
// alike.  The kept positions ascend along the slots, so the positions matched to slot j are the contiguous
// range (mid(j-1), mid(j)] with mid(j) = floor((kept_pos[j] + kept_pos[j+1]) / 2): no matching pass is
// needed.  One workgroup per (segment, kv head, part of the slot list); a row group of a wavefront takes a slot
// and sums its range in ascending order (long ranges: the whole wavefront, 64/LPR rows per load instruction, the
// groups' sums added in a fixed order).  Every row of K and V is read exactly once per launch.
template <int LPR, bool BF16>
__global__ void __launch_bounds__(256)
merge_position_kernel(int nparts, int Hkv, int L, int N, int row_bytes, const unsigned char* __restrict__ k,
                      Strides ks, const unsigned char* __restrict__ v, Strides vs, int esize,
                      const int64_t* __restrict__ seg_off, const int32_t* __restrict__ caps,
                      const int32_t* __restrict__ lens, const int32_t* __restrict__ kept_pos,
                      unsigned char* __restrict__ kc, unsigned char* __restrict__ vc) {
    constexpr int RPI = kWave / LPR;         // rows per wavefront-wide load
    constexpr int EPL = BF16 ? 8 : 4;        // elements per lane
    const int part = blockIdx.x % nparts;
    const int h = (blockIdx.x / nparts) % Hkv, seg = blockIdx.x / (nparts * Hkv);
    const int len = lens[seg];
    const int per = (len + nparts - 1) / nparts;
    const int j0 = part * per, j1 = min(len, j0 + per);
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave;
    const int sub = lane % LPR, rg = lane / LPR;
    const int b = seg / L, l = seg % L;
    const int64_t off = seg_off[seg];
    const int cap = caps[seg];
    const int32_t* kp = kept_pos + off;
    const unsigned char* kb = k + (ks.b * b + ks.l * l + ks.h * h) * (int64_t)esize + sub * 16;
    const unsigned char* vb = v + (vs.b * b + vs.l * l + vs.h * h) * (int64_t)esize + sub * 16;
    const int64_t kstep = ks.n * (int64_t)esize, vstep = vs.n * (int64_t)esize;
    // accumulate one row chunk (16 bytes of this lane) into fp32 sums
    auto add16 = [](float (&acc)[EPL], const uint4& r) {
        const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            if constexpr (BF16) {
                acc[2 * x] += __uint_as_float(w[x] << 16);
                acc[2 * x + 1] += __uint_as_float(w[x] & 0xffff0000u);
            } else {
                acc[x] += __uint_as_float(w[x]);
            }
        }
    };
    auto store_mean = [&](int j, const float (&ka)[EPL], const float (&va)[EPL], float cnt) {
        const int64_t dst = (off * Hkv + (int64_t)h * cap + j) * row_bytes + sub * 16;
        if constexpr (BF16) {
            uint32_t ko[4], vo[4];
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                ko[x] = (uint32_t)f32_to_bf16(ka[2 * x] / cnt) | ((uint32_t)f32_to_bf16(ka[2 * x + 1] / cnt) << 16);
                vo[x] = (uint32_t)f32_to_bf16(va[2 * x] / cnt) | ((uint32_t)f32_to_bf16(va[2 * x + 1] / cnt) << 16);
            }
            *(uint4*)(kc + dst) = make_uint4(ko[0], ko[1], ko[2], ko[3]);
            *(uint4*)(vc + dst) = make_uint4(vo[0], vo[1], vo[2], vo[3]);
        } else {
            *(uint4*)(kc + dst) = make_uint4(__float_as_uint(ka[0] / cnt), __float_as_uint(ka[1] / cnt),
                                             __float_as_uint(ka[2] / cnt), __float_as_uint(ka[3] / cnt));
            *(uint4*)(vc + dst) = make_uint4(__float_as_uint(va[0] / cnt), __float_as_uint(va[1] / cnt),
                                             __float_as_uint(va[2] / cnt), __float_as_uint(va[3] / cnt));
        }
    };
    // A wavefront takes RPI consecutive slots at a time, one per row group (LPR lanes = one row): a group walks
    // the range of its slot two rows deep and holds the whole sums, no exchange between lanes.  A range longer
    // than kLongRange rows (a layer that keeps little of a long prompt) is walked by the whole wavefront
    // afterwards, RPI rows per load instruction, and the groups' sums are added in a fixed order.
    constexpr int kLongRange = 32;
    for (int jb = j0 + wv * RPI; jb < j1; jb += 4 * RPI) {
        const int j = jb + rg;
        const bool act = j < j1;
        int lo = 0, hi = 0;
        if (act) {
            const int pj = kp[j];
            lo = j == 0 ? 0 : (kp[j - 1] + pj) / 2 + 1;
            hi = j == len - 1 ? N : (pj + kp[j + 1]) / 2 + 1;
        }
        const bool is_long = act && hi - lo > kLongRange;
        const unsigned long long longmask = __builtin_amdgcn_ballot_w64(is_long && sub == 0);
        if (act && !is_long) {
            float ka[EPL], va[EPL];
#pragma unroll
            for (int x = 0; x < EPL; ++x) { ka[x] = 0.f; va[x] = 0.f; }
            for (int m = lo; m < hi; m += 2) {
                uint4 r[4];
                r[2] = r[3] = make_uint4(0, 0, 0, 0);     // zero bits are 0.0 in both formats
                r[0] = *(const uint4*)(kb + kstep * m);
                r[1] = *(const uint4*)(vb + vstep * m);
                if (m + 1 < hi) { r[2] = *(const uint4*)(kb + kstep * (m + 1)); r[3] = *(const uint4*)(vb + vstep * (m + 1)); }
                add16(ka, r[0]); add16(va, r[1]); add16(ka, r[2]); add16(va, r[3]);
            }
            store_mean(j, ka, va, (float)(hi - lo));      // >= 1 row: the range holds the kept position itself
        }
        for (unsigned long long lm = longmask; lm; lm &= lm - 1) {
            const int src = __builtin_ctzll(lm);          // first lane of the group that owns the long slot
            const int jl = jb + src / LPR;
            const int llo = __shfl(lo, src, kWave), lhi = __shfl(hi, src, kWave);
            float ka[EPL], va[EPL];
#pragma unroll
            for (int x = 0; x < EPL; ++x) { ka[x] = 0.f; va[x] = 0.f; }
            for (int m0 = llo; m0 < lhi; m0 += 2 * RPI) {
                const int ma = m0 + rg, mb = m0 + RPI + rg;
                uint4 r[4];
                r[0] = r[1] = r[2] = r[3] = make_uint4(0, 0, 0, 0);
                if (ma < lhi) { r[0] = *(const uint4*)(kb + kstep * ma); r[1] = *(const uint4*)(vb + vstep * ma); }
                if (mb < lhi) { r[2] = *(const uint4*)(kb + kstep * mb); r[3] = *(const uint4*)(vb + vstep * mb); }
                add16(ka, r[0]); add16(va, r[1]); add16(ka, r[2]); add16(va, r[3]);
            }
#pragma unroll
            for (int sh = LPR; sh < kWave; sh <<= 1)
#pragma unroll
                for (int x = 0; x < EPL; ++x) {
                    ka[x] += __shfl_xor(ka[x], sh, kWave);
                    va[x] += __shfl_xor(va[x], sh, kWave);
                }
            if (rg == 0) store_mean(jl, ka, va, (float)(lhi - llo));
        }
    }
}

size_t compact_ws_bytes(const pkv_shape&) { return 0; }

hipError_t launch_merge_position(const pkv_shape& s, const void* k, Strides ks, const void* v, Strides vs,
                                 const int64_t* seg_off, const int32_t* caps, const int32_t* kept_pos,
                                 const int32_t* lens, void* kc, void* vc, hipStream_t st) {
    const int nseg = s.B * s.L;
    const bool bf16 = s.dtype == PKV_BF16;
    const int esize = bf16 ? 2 : 4;
    const int row_bytes = s.D * esize;
    const int lpr = row_bytes / 16;
    // enough workgroups to fill the chip, but few: a workgroup's start (segment state, kept positions) is a chain
    // of dependent loads, and more, smaller workgroups were slower at every size measured
    const int want = s.N <= 1024 ? 2048 : 1024;
    int nparts = (want + nseg * s.Hkv - 1) / (nseg * s.Hkv);
    nparts = nparts < 1 ? 1 : (nparts > 8 ? 8 : nparts);
    dim3 grid((uint32_t)((size_t)nparts * s.Hkv * nseg));
#define PKV_MERGE(LPR, BF)                                                                                   \
    hipLaunchKernelGGL((merge_position_kernel<LPR, BF>), grid, dim3(256), 0, st, nparts, s.Hkv, s.L, s.N,     \
                       row_bytes, (const unsigned char*)k, ks, (const unsigned char*)v, vs, esize, seg_off,  \
                       caps, lens, kept_pos, (unsigned char*)kc, (unsigned char*)vc)
    if (bf16 && lpr == 8) PKV_MERGE(8, true);
    else if (bf16) PKV_MERGE(16, true);
    else if (lpr == 16) PKV_MERGE(16, false);
    else PKV_MERGE(32, false);
#undef PKV_MERGE
    return hipGetLastError();
}

// Workgroups per (segment, kv head): one per 64-row chunk up to 16 chunks (1024 rows), made odd.  The hardware
// deals consecutive workgroups out to the eight XCDs in turn; with an even count -- 16 above all -- chunk c of
// every (segment, head) lands on the same XCD, and since most segments keep few rows the XCDs of the high
// chunk indices see hardly any work (measured with 16: 2.3 instead of 4.3 TB/s from N = 1000 on).
static int gather_chunks(int N) {
    const int all_chunks = (N + 63) / 64;
    const int nchunk = all_chunks < 16 ? all_chunks : 16;
    return nchunk | 1;
}

hipError_t launch_compact(const pkv_shape& s, const void* k, Strides ks, const void* v, Strides vs,
                          const int32_t* order, const int32_t* lengths, int decode_capacity,
                          int64_t* seg_off, int32_t* caps, void* kc, void* vc, int32_t* kept_pos,
                          int32_t* lens, void*, hipStream_t st) {
    const int nseg = s.B * s.L;
    const int esize = s.dtype == PKV_F32 ? 4 : 2;
    const int row_bytes = s.D * esize;
    const int lpr = row_bytes / 16;
    const int nchunk = gather_chunks(s.N);
    dim3 grid((uint32_t)((size_t)nchunk * s.Hkv * nseg));
    static_assert((size_t)kMaxN * 5 + 256 <= 64 * 1024, "the position list and the flags of the longest prompt fit the default LDS limit");
    const size_t lds = (size_t)s.N * 4 + (size_t)((s.N + 3) / 4) * 4;
    const bool ntl = 2 * (size_t)nseg * s.Hkv * s.N * row_bytes >= ((size_t)1 << 31);   // K and V: 2 GiB or more
#define PKV_FUSED(LPR, NTL)                                                                                        \
    hipLaunchKernelGGL((compact_fused_kernel<LPR, NTL>), grid, dim3(256), lds, st, s.N, nchunk, s.Hkv, s.L, row_bytes, \
                       (const unsigned char*)k, ks, (const unsigned char*)v, vs, esize, order, lengths,            \
                       decode_capacity, seg_off, caps, lens, kept_pos, (unsigned char*)kc, (unsigned char*)vc)
    if (ntl) {
        if (lpr == 8) PKV_FUSED(8, true);
        else if (lpr == 16) PKV_FUSED(16, true);
        else PKV_FUSED(32, true);
    } else {
        if (lpr == 8) PKV_FUSED(8, false);
        else if (lpr == 16) PKV_FUSED(16, false);
        else PKV_FUSED(32, false);
    }
#undef PKV_FUSED
    return hipGetLastError();
}

}  // namespace pkv
