// Stage 4a: gather the kept K/V rows of every layer into the ragged per-layer cache (Sec. 3.2: the
// top R_l proportion is retained in each head of layer l; all heads of a layer share one index set).
//
//  compact_plan_kernel   one workgroup per (sequence, layer): segment offset (sum of the capacities of
//                        the segments before it), capacity, and the kept positions in ascending order
//                        (flag array in LDS -> exclusive scan -> scatter).
//  compact_gather_kernel streams whole rows (16 B per lane) from K/V into the segment.  Pure HBM traffic.
#include "pkv_common.hpp"

namespace pkv {

__device__ __forceinline__ int block_excl_scan_i32(int v, int* s_wave, int& total) {
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave, nw = blockDim.x / kWave;
    int incl = v;
    for (int d = 1; d < kWave; d <<= 1) {
        const int up = __shfl_up(incl, d, kWave);
        if (lane >= d) incl += up;
    }
    __syncthreads();  // s_wave may still be in use by a previous call
    if (lane == kWave - 1) s_wave[wv] = incl;
    __syncthreads();
    int base = 0, tot = 0;
    for (int w = 0; w < nw; ++w) {
        const int t = s_wave[w];
        if (w < wv) base += t;
        tot += t;
    }
    total = tot;
    return base + incl - v;
}

__global__ void compact_plan_kernel(int N, int nseg, const int32_t* __restrict__ order,
                                    const int32_t* __restrict__ lengths, int decode_capacity,
                                    int64_t* __restrict__ seg_off, int32_t* __restrict__ caps,
                                    int32_t* __restrict__ kept_pos, int32_t* __restrict__ lens) {
    extern __shared__ unsigned char s_flag[];  // N flags
    __shared__ int s_wave[16];
    __shared__ long long s_off[16];
    const int tid = threadIdx.x, nt = blockDim.x, seg = blockIdx.x;
    const int lane = tid & (kWave - 1), wv = tid / kWave, nw = nt / kWave;

    // token offset of this segment = sum of (length + capacity) of all segments before it
    long long acc = 0;
    for (int i = tid; i < seg; i += nt) acc += (long long)lengths[i] + decode_capacity;
    for (int d = 32; d > 0; d >>= 1) {
        const uint32_t lo = __shfl_xor((uint32_t)acc, d, kWave);
        const uint32_t hi = __shfl_xor((uint32_t)((unsigned long long)acc >> 32), d, kWave);
        acc += (long long)(((unsigned long long)hi << 32) | lo);
    }
    if (lane == 0) s_off[wv] = acc;
    for (int i = tid; i < N; i += nt) s_flag[i] = 0;
    __syncthreads();
    long long off = 0;
    for (int w = 0; w < nw; ++w) off += s_off[w];

    int klen = lengths[seg];
    klen = klen < 0 ? 0 : (klen > N ? N : klen);
    const int32_t* ord = order + (size_t)seg * N;
    for (int j = tid; j < klen; j += nt) {
        const int pos = ord[j];
        if (pos >= 0 && pos < N) s_flag[pos] = 1;
    }
    __syncthreads();
    const int E = (N + nt - 1) / nt;
    const int lo = tid * E, hi = min(lo + E, N);
    int cnt = 0;
    for (int i = lo; i < hi; ++i) cnt += s_flag[i];
    int total;
    int at = block_excl_scan_i32(cnt, s_wave, total);
    for (int i = lo; i < hi; ++i)
        if (s_flag[i]) kept_pos[off + at++] = i;
    if (tid == 0) {
        seg_off[seg] = off;
        caps[seg] = klen + decode_capacity;
        lens[seg] = klen;
    }
}

// A workgroup copies kRows kept rows of one (segment, kv head) at a time, K and V; `nchunk` workgroups share
// a (segment, kv head) and stride over its chunks, so no workgroup is launched for rows that were not kept.
// LPR lanes cover a row with one 16-byte load each, so a wavefront moves 64/LPR whole rows per instruction.
template <int LPR>
__global__ void __launch_bounds__(256)
compact_gather_kernel(int nchunk, int Hkv, int L, int row_bytes, const unsigned char* __restrict__ k, Strides ks,
                      const unsigned char* __restrict__ v, Strides vs, int esize,
                      const int64_t* __restrict__ seg_off, const int32_t* __restrict__ caps,
                      const int32_t* __restrict__ lens, const int32_t* __restrict__ kept_pos,
                      unsigned char* __restrict__ kc, unsigned char* __restrict__ vc) {
    constexpr int kRows = 64;
    constexpr int RPI = 256 / LPR;  // rows per workgroup-wide instruction
    const int h = (blockIdx.x / nchunk) % Hkv, seg = blockIdx.x / (nchunk * Hkv);
    const int len = lens[seg];
    if ((int)(blockIdx.x % nchunk) * kRows >= len) return;
    const int b = seg / L, l = seg % L;
    const int64_t off = seg_off[seg];
    const int cap = caps[seg];
    const int sub = threadIdx.x % LPR, rsel = threadIdx.x / LPR;
    const unsigned char* kb = k + (ks.b * b + ks.l * l + ks.h * h) * (int64_t)esize;
    const unsigned char* vb = v + (vs.b * b + vs.l * l + vs.h * h) * (int64_t)esize;
    const int64_t dst0 = (off * Hkv + (int64_t)h * cap) * row_bytes;
    for (int r0 = (int)(blockIdx.x % nchunk) * kRows; r0 < len; r0 += nchunk * kRows) {
        uint4 kr[kRows / RPI], vr[kRows / RPI];
#pragma unroll
        for (int i = 0; i < kRows / RPI; ++i) {
            const int r = r0 + i * RPI + rsel;
            kr[i] = vr[i] = make_uint4(0, 0, 0, 0);   // (defined on every path: the arrays stay in registers)
            if (r < len) {
                const int pos = kept_pos[off + r];
                kr[i] = *(const uint4*)(kb + ks.n * pos * (int64_t)esize + sub * 16);
                vr[i] = *(const uint4*)(vb + vs.n * pos * (int64_t)esize + sub * 16);
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

hipError_t launch_compact(const pkv_shape& s, const void* k, Strides ks, const void* v, Strides vs,
                          const int32_t* order, const int32_t* lengths, int decode_capacity,
                          int64_t* seg_off, int32_t* caps, void* kc, void* vc, int32_t* kept_pos,
                          int32_t* lens, void*, hipStream_t st) {
    const int nseg = s.B * s.L;
    const int nt = s.N > 2048 ? 1024 : 256;
    hipLaunchKernelGGL(compact_plan_kernel, dim3(nseg), dim3(nt), (size_t)s.N, st, s.N, nseg, order,
                       lengths, decode_capacity, seg_off, caps, kept_pos, lens);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int esize = s.dtype == PKV_F32 ? 4 : 2;
    const int row_bytes = s.D * esize;
    const int lpr = row_bytes / 16;
    // workgroups per (segment, kv head): one per chunk up to 16 (1024 rows); for longer prompts a workgroup
    // walks further chunks -- most segments keep a small part of a long prompt, and workgroups that find
    // nothing to do are not free (measured at N = 8192: 0.34 -> 0.27 ms; fewer than one workgroup per chunk
    // at N = 680 is slower: the copies of a workgroup are one dependent chain)
    const int all_chunks = (s.N + 63) / 64;
    const int nchunk = all_chunks < 16 ? all_chunks : 16;
    dim3 grid((uint32_t)((size_t)nchunk * s.Hkv * nseg));
#define PKV_GATHER(LPR)                                                                                  \
    hipLaunchKernelGGL(compact_gather_kernel<LPR>, grid, dim3(256), 0, st, nchunk, s.Hkv, s.L, row_bytes,       \
                       (const unsigned char*)k, ks, (const unsigned char*)v, vs, esize, seg_off, caps,  \
                       lens, kept_pos, (unsigned char*)kc, (unsigned char*)vc)
    if (lpr == 8) PKV_GATHER(8);
    else if (lpr == 16) PKV_GATHER(16);
    else PKV_GATHER(32);
#undef PKV_GATHER
    return hipGetLastError();
}

}  // namespace pkv
