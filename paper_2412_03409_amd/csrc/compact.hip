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

// One workgroup copies kRows kept rows of one (segment, kv head) for K and V.  LPR lanes cover a row
// with one 16-byte load each, so a wavefront moves 64/LPR whole rows per instruction.
template <int LPR>
__global__ void __launch_bounds__(256)
compact_gather_kernel(int nchunk, int Hkv, int L, int row_bytes, const unsigned char* __restrict__ k, Strides ks,
                      const unsigned char* __restrict__ v, Strides vs, int esize,
                      const int64_t* __restrict__ seg_off, const int32_t* __restrict__ caps,
                      const int32_t* __restrict__ lens, const int32_t* __restrict__ kept_pos,
                      unsigned char* __restrict__ kc, unsigned char* __restrict__ vc) {
    constexpr int kRows = 64;
    constexpr int RPI = 256 / LPR;  // rows per workgroup-wide instruction
    const int chunk = blockIdx.x % nchunk;
    const int h = (blockIdx.x / nchunk) % Hkv, seg = blockIdx.x / (nchunk * Hkv);
    const int len = lens[seg];
    const int r0 = chunk * kRows;
    if (r0 >= len) return;
    const int b = seg / L, l = seg % L;
    const int64_t off = seg_off[seg];
    const int cap = caps[seg];
    const int sub = threadIdx.x % LPR, rsel = threadIdx.x / LPR;
    const unsigned char* kb = k + (ks.b * b + ks.l * l + ks.h * h) * (int64_t)esize;
    const unsigned char* vb = v + (vs.b * b + vs.l * l + vs.h * h) * (int64_t)esize;
    const int64_t dst0 = (off * Hkv + (int64_t)h * cap) * row_bytes;
    uint4 kr[kRows / RPI], vr[kRows / RPI];
#pragma unroll
    for (int i = 0; i < kRows / RPI; ++i) {
        const int r = r0 + i * RPI + rsel;
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

size_t compact_ws_bytes(const pkv_shape&) { return 0; }

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
    const int nchunk = (s.N + 63) / 64;
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
