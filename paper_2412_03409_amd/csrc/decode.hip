// Stage 4b: one decode step over the ragged compressed cache (Sec. 3.1: the newest token's query
// interacts with the cached KV vectors of every layer).
//
//  decode_attn_kernel     split-KV attention.  The work is cut into equal units of kDecodeChunk (64)
//                         cached tokens of one (sequence, layer, kv head); a wavefront owns one unit at a
//                         time and a fixed grid walks all units round-robin, so ragged layer lengths do
//                         not unbalance the chip.  A wavefront issues all K and V loads of its unit up
//                         front (16 B per lane, whole rows, fully coalesced), then does the dot products,
//                         a block softmax and the weighted V sum in registers, for every query head that
//                         shares the kv head, so each cached byte is read from HBM exactly once.
//                         The new token's k/v (append) are taken from k_new/v_new in place of the slot
//                         they are written to, so no unit ever reads a slot written in the same launch.
//  decode_combine_kernel  merges the per-unit partial results (max, sum, weighted V) of every query
//                         head, writes the output and publishes the new lens.
//
// The unit table (chunks per segment, prefix-summed) is rebuilt from lens in LDS by every workgroup:
// it is a few hundred integers, cheaper than another dependent launch.
#include "pkv_common.hpp"

namespace pkv {

struct DecodeParams {
    int B, L, l0, nl, H, Hkv, D, grp, append;
    const unsigned char* q;       // [B,L,H,D]
    const unsigned char* k_new;   // [B,L,Hkv,D]
    const unsigned char* v_new;
    const float* scale;           // [L]
    unsigned char* kc;
    unsigned char* vc;
    const int64_t* seg_off;       // [B,L]
    const int32_t* caps;          // [B,L]
    int32_t* lens;                // [B,L]
    unsigned char* out;           // [B,L,H,D]
    int32_t* plan;                // ws: pre[nseg+1], efflen[nseg]
    float* part;                  // ws: [unit][G][D+2]
    long long max_units;          // capacity of `part` in (unit) entries of G heads
};

template <bool BF16>
__device__ __forceinline__ void unpack16(const uint4& r, float* f) {
    if constexpr (BF16) {
        f[0] = __uint_as_float(r.x << 16); f[1] = __uint_as_float(r.x & 0xffff0000u);
        f[2] = __uint_as_float(r.y << 16); f[3] = __uint_as_float(r.y & 0xffff0000u);
        f[4] = __uint_as_float(r.z << 16); f[5] = __uint_as_float(r.z & 0xffff0000u);
        f[6] = __uint_as_float(r.w << 16); f[7] = __uint_as_float(r.w & 0xffff0000u);
    } else {
        f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y);
        f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
    }
}

// Exclusive scan of the chunk counts of all segments into s_pre[0..nseg]; s_pre[nseg] = total.
__device__ __forceinline__ void build_plan(const DecodeParams& p, int nseg, int* s_pre, int* s_wave) {
    const int tid = threadIdx.x, nt = blockDim.x;
    const int lane = tid & (kWave - 1), wv = tid / kWave, nw = nt / kWave;
    const int E = (nseg + nt - 1) / nt;
    const int lo = tid * E, hi = min(lo + E, nseg);
    int cnt = 0;
    for (int i = lo; i < hi; ++i) {
        const int sl = (i / p.nl) * p.L + p.l0 + i % p.nl;
        int len = p.lens[sl];
        if (p.append && len < p.caps[sl]) len += 1;
        const int nch = (len + kDecodeChunk - 1) / kDecodeChunk;
        s_pre[i] = cnt;  // thread-local exclusive, rebased below
        cnt += nch;
    }
    int incl = cnt;
    for (int d = 1; d < kWave; d <<= 1) {
        const int up = __shfl_up(incl, d, kWave);
        if (lane >= d) incl += up;
    }
    if (lane == kWave - 1) s_wave[wv] = incl;
    __syncthreads();
    int base = 0, tot = 0;
    for (int w = 0; w < nw; ++w) {
        const int t = s_wave[w];
        if (w < wv) base += t;
        tot += t;
    }
    const int excl = base + incl - cnt;
    for (int i = lo; i < hi; ++i) s_pre[i] += excl;
    if (tid == 0) s_pre[nseg] = tot;
    __syncthreads();
}

template <bool BF16, int LPR, int G>
__global__ void __launch_bounds__(256)
decode_attn_kernel(DecodeParams p) {
    constexpr int EPL = BF16 ? 8 : 4;            // elements per lane (16 bytes)
    constexpr int RPI = kWave / LPR;             // rows per wavefront-wide load instruction
    constexpr int NI = (kDecodeChunk / RPI) < 16 ? (kDecodeChunk / RPI) : 16;  // loads in flight
    constexpr int SB = NI * RPI;                 // rows per sub-block
    constexpr int NSB = kDecodeChunk / SB;
    constexpr int ESZ = BF16 ? 2 : 4;
    extern __shared__ int s_pre[];               // nseg + 1
    __shared__ int s_wave[4];

    const int nseg = p.B * p.nl;
    build_plan(p, nseg, s_pre, s_wave);
    const int total_chunks = s_pre[nseg];
    if (blockIdx.x == 0) {  // publish the plan for the combine kernel
        for (int i = threadIdx.x; i <= nseg; i += blockDim.x) p.plan[i] = s_pre[i];
        for (int i = threadIdx.x; i < nseg; i += blockDim.x) {
            const int sl = (i / p.nl) * p.L + p.l0 + i % p.nl;
            int len = p.lens[sl];
            if (p.append && len < p.caps[sl]) len += 1;
            p.plan[nseg + 1 + i] = len;
        }
    }

    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave;
    const int sub = lane % LPR, rg = lane / LPR;
    const int HU = p.H / G;                      // head units per segment
    const long long U = (long long)total_chunks * HU;
    const long long GW = (long long)gridDim.x * (blockDim.x / kWave);
    const int row_bytes = p.D * ESZ;
    const float LOG2E = 1.4426950408889634f;

    for (long long u = (long long)blockIdx.x * (blockDim.x / kWave) + wv; u < U && u < p.max_units; u += GW) {
        const int ci = (int)(u / HU), hu = (int)(u % HU);
        // segment that owns global chunk ci: largest i with s_pre[i] <= ci
        int a = 0, e = nseg - 1;
        while (a < e) {
            const int m = (a + e + 1) >> 1;
            if (s_pre[m] <= ci) a = m; else e = m - 1;
        }
        const int i_seg = a, c = ci - s_pre[a];
        const int b = i_seg / p.nl, l = p.l0 + i_seg % p.nl, sl = b * p.L + l;
        const int len_old = p.lens[sl];
        const int cap = p.caps[sl];
        const bool app = p.append && len_old < cap;
        const int len = len_old + (app ? 1 : 0);
        const int kvh = (hu * G) / p.grp;
        const bool writer = app && ((hu * G) % p.grp == 0);
        const int64_t segbase = (p.seg_off[sl] * p.Hkv + (int64_t)kvh * cap) * row_bytes;
        const unsigned char* kbase = p.kc + segbase;
        const unsigned char* vbase = p.vc + segbase;
        const int64_t newrow = ((int64_t)sl * p.Hkv + kvh) * row_bytes;
        const float qs = p.scale[l] * LOG2E;

        float o[G][EPL], mrun[G], srun[G];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            mrun[g] = -INFINITY; srun[g] = 0.f;
#pragma unroll
            for (int x = 0; x < EPL; ++x) o[g][x] = 0.f;
        }

#pragma unroll
        for (int sb = 0; sb < NSB; ++sb) {
            const int r0 = c * kDecodeChunk + sb * SB;
            if (r0 >= len) break;
            uint4 kr[NI], vr[NI];
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                const int r = r0 + i * RPI + rg;
                kr[i] = make_uint4(0, 0, 0, 0); vr[i] = make_uint4(0, 0, 0, 0);
                if (r < len) {
                    const bool isnew = app && r == len_old;
                    const unsigned char* kp = isnew ? p.k_new + newrow : kbase + (int64_t)r * row_bytes;
                    const unsigned char* vp = isnew ? p.v_new + newrow : vbase + (int64_t)r * row_bytes;
                    kr[i] = *(const uint4*)(kp + sub * 16);
                    vr[i] = *(const uint4*)(vp + sub * 16);
                    if (isnew && writer) {
                        *(uint4*)(p.kc + segbase + (int64_t)r * row_bytes + sub * 16) = kr[i];
                        *(uint4*)(p.vc + segbase + (int64_t)r * row_bytes + sub * 16) = vr[i];
                    }
                }
            }
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const int h = hu * G + g;
                float qf[EPL];
                {
                    const uint4 qr = *(const uint4*)(p.q + ((int64_t)sl * p.H + h) * row_bytes + sub * 16);
                    unpack16<BF16>(qr, qf);
#pragma unroll
                    for (int x = 0; x < EPL; ++x) qf[x] *= qs;
                }
                float s[NI];
                float mx = -INFINITY;
#pragma unroll
                for (int i = 0; i < NI; ++i) {
                    float kf[EPL];
                    unpack16<BF16>(kr[i], kf);
                    float d = 0.f;
#pragma unroll
                    for (int x = 0; x < EPL; ++x) d = fmaf(qf[x], kf[x], d);
#pragma unroll
                    for (int sh = 1; sh < LPR; sh <<= 1) d += __shfl_xor(d, sh, kWave);
                    const int r = r0 + i * RPI + rg;
                    s[i] = r < len ? d : -INFINITY;
                    mx = fmaxf(mx, s[i]);
                }
#pragma unroll
                for (int sh = LPR; sh < kWave; sh <<= 1) mx = fmaxf(mx, __shfl_xor(mx, sh, kWave));
                // r0 < len, so at least one row of the sub-block is valid and mx is finite
                const float mnew = fmaxf(mrun[g], mx);
                const float corr = __builtin_amdgcn_exp2f(mrun[g] - mnew);  // exp2(-inf) = 0 on the first sub-block
                float ps = 0.f;
#pragma unroll
                for (int x = 0; x < EPL; ++x) o[g][x] *= corr;
#pragma unroll
                for (int i = 0; i < NI; ++i) {
                    const float pr = __builtin_amdgcn_exp2f(s[i] - mnew);
                    ps += pr;
                    float vf[EPL];
                    unpack16<BF16>(vr[i], vf);
#pragma unroll
                    for (int x = 0; x < EPL; ++x) o[g][x] = fmaf(pr, vf[x], o[g][x]);
                }
                srun[g] = srun[g] * corr + ps;  // per row group; merged across groups below
                mrun[g] = mnew;
            }
        }
        // merge the RPI row groups (they share mrun) and store the unit's partial result
#pragma unroll
        for (int g = 0; g < G; ++g) {
#pragma unroll
            for (int sh = LPR; sh < kWave; sh <<= 1) {
                srun[g] += __shfl_xor(srun[g], sh, kWave);
#pragma unroll
                for (int x = 0; x < EPL; ++x) o[g][x] += __shfl_xor(o[g][x], sh, kWave);
            }
            if (rg == 0) {
                float* dst = p.part + ((size_t)u * G + g) * (size_t)(p.D + 2);
                float4* d4 = (float4*)(dst + sub * EPL);
                d4[0] = make_float4(o[g][0], o[g][1], o[g][2], o[g][3]);
                if constexpr (EPL == 8) d4[1] = make_float4(o[g][4], o[g][5], o[g][6], o[g][7]);
                if (sub == 0) { dst[p.D] = mrun[g]; dst[p.D + 1] = srun[g]; }
            }
        }
    }
}

// One thread per (segment, query head, d).  Reads only the published plan, never lens, so that the
// lens update below cannot race with another workgroup of the same launch.
template <bool BF16, int G>
__global__ void __launch_bounds__(256)
decode_combine_kernel(DecodeParams p) {
    const int nseg = p.B * p.nl;
    const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const int d = (int)(gid % p.D);
    const long long sh = gid / p.D;
    if (sh >= (long long)nseg * p.H) return;
    const int h = (int)(sh % p.H), i_seg = (int)(sh / p.H);
    const int b = i_seg / p.nl, l = p.l0 + i_seg % p.nl, sl = b * p.L + l;
    const int HU = p.H / G, hu = h / G, g = h % G;
    const int c0 = p.plan[i_seg], nch = p.plan[i_seg + 1] - c0;
    float M = -INFINITY;
    for (int c = 0; c < nch; ++c) {
        const long long u = (long long)(c0 + c) * HU + hu;
        M = fmaxf(M, p.part[((size_t)u * G + g) * (size_t)(p.D + 2) + p.D]);
    }
    float num = 0.f, den = 0.f;
    for (int c = 0; c < nch; ++c) {
        const long long u = (long long)(c0 + c) * HU + hu;
        const float* src = p.part + ((size_t)u * G + g) * (size_t)(p.D + 2);
        const float w = exp2f(src[p.D] - M);
        num = fmaf(w, src[d], num);
        den = fmaf(w, src[p.D + 1], den);
    }
    const float r = nch > 0 ? num / den : 0.f;
    const size_t oi = ((size_t)sl * p.H + h) * p.D + d;
    if constexpr (BF16) ((bf16_t*)p.out)[oi] = f32_to_bf16(r); else ((float*)p.out)[oi] = r;
    if (h == 0 && d == 0) p.lens[sl] = p.plan[nseg + 1 + i_seg];
}

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

static long long decode_max_chunks(const pkv_shape& s, int64_t cache_tokens) {
    return cache_tokens / kDecodeChunk + (long long)s.B * s.L;
}
static size_t decode_plan_bytes(const pkv_shape& s) {
    return align_up((size_t)(2 * (size_t)s.B * s.L + 1) * sizeof(int32_t), 256);
}

size_t decode_ws_bytes(const pkv_shape& s, int64_t cache_tokens) {
    // one partial (D+2 floats) per (chunk, query head)
    return decode_plan_bytes(s) +
           (size_t)decode_max_chunks(s, cache_tokens) * s.H * (size_t)(s.D + 2) * sizeof(float);
}

static int pick_group(int grp) { return grp % 8 == 0 ? 8 : grp % 4 == 0 ? 4 : grp % 2 == 0 ? 2 : 1; }

template <bool BF16, int LPR, int G>
static hipError_t launch_decode_t(const DecodeParams& p, int nblk, int nblk_combine, size_t lds,
                                  hipStream_t st) {
    hipLaunchKernelGGL((decode_attn_kernel<BF16, LPR, G>), dim3(nblk), dim3(256), lds, st, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((decode_combine_kernel<BF16, G>), dim3(nblk_combine), dim3(256), 0, st, p);
    return hipGetLastError();
}

template <bool BF16, int LPR>
static hipError_t launch_decode_g(const DecodeParams& p, int G, int nblk, int nblk_combine, size_t lds,
                                  hipStream_t st) {
    switch (G) {
        case 8: return launch_decode_t<BF16, LPR, 8>(p, nblk, nblk_combine, lds, st);
        case 4: return launch_decode_t<BF16, LPR, 4>(p, nblk, nblk_combine, lds, st);
        case 2: return launch_decode_t<BF16, LPR, 2>(p, nblk, nblk_combine, lds, st);
        default: return launch_decode_t<BF16, LPR, 1>(p, nblk, nblk_combine, lds, st);
    }
}

hipError_t launch_decode(const pkv_shape& s, int l0, int l1, const void* q, const void* k_new,
                         const void* v_new, const float* scale, void* kc, void* vc,
                         const int64_t* seg_off, const int32_t* caps, int32_t* lens, void* out,
                         int64_t cache_tokens, void* ws, hipStream_t st) {
    DecodeParams p;
    p.B = s.B; p.L = s.L; p.l0 = l0; p.nl = l1 - l0; p.H = s.H; p.Hkv = s.Hkv; p.D = s.D;
    p.grp = s.H / s.Hkv; p.append = k_new != nullptr;
    p.q = (const unsigned char*)q; p.k_new = (const unsigned char*)k_new;
    p.v_new = (const unsigned char*)v_new; p.scale = scale;
    p.kc = (unsigned char*)kc; p.vc = (unsigned char*)vc; p.seg_off = seg_off; p.caps = caps;
    p.lens = lens; p.out = (unsigned char*)out;
    p.plan = (int32_t*)ws;
    p.part = (float*)((unsigned char*)ws + decode_plan_bytes(s));
    const int G = pick_group(p.grp);
    p.max_units = decode_max_chunks(s, cache_tokens) * (s.H / G);
    const int nseg = s.B * p.nl;
    const size_t lds = (size_t)(nseg + 1) * sizeof(int);
    long long want = (p.max_units + 3) / 4;
    const int nblk = (int)(want < 1 ? 1 : (want > 1024 ? 1024 : want));
    const long long nthr = (long long)nseg * s.H * s.D;
    const int nblk_combine = (int)((nthr + 255) / 256);
    const bool bf16 = s.dtype == PKV_BF16;
    const int lpr = s.D * (bf16 ? 2 : 4) / 16;
    if (bf16) {
        if (lpr == 8) return launch_decode_g<true, 8>(p, G, nblk, nblk_combine, lds, st);
        return launch_decode_g<true, 16>(p, G, nblk, nblk_combine, lds, st);
    }
    if (lpr == 16) return launch_decode_g<false, 16>(p, G, nblk, nblk_combine, lds, st);
    return launch_decode_g<false, 32>(p, G, nblk, nblk_combine, lds, st);
}

}  // namespace pkv
