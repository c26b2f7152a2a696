// Stage 4b: one decode step over the ragged compressed cache (Sec. 3.1: the newest token's query
// interacts with the cached KV vectors of every layer).  ONE kernel per step:
//
//  decode_attn_kernel   a workgroup of a few wavefronts owns one (sequence, layer, kv head) -- or a
//                       sub-group of G of its query heads -- and its wavefronts take the segment's
//                       64-token chunks round-robin.  A wavefront issues all K and V loads of a chunk up
//                       front (16 B per lane, whole rows, fully coalesced), then does
//                       the dot products, a block softmax and the weighted V sum in registers for every
//                       query head of the group, so each cached byte is read from HBM once per group.
//                       The wavefronts' (max, sum, weighted V) are merged through LDS and the output is
//                       written directly: no partial results ever go to HBM.
//
// Append: the new token's k/v are taken from k_new/v_new in place of the slot they are written to, so
// no wavefront reads a slot that is written in the same launch.
//
// lens is advanced inside the same launch without a second kernel: every workgroup reads the old
// length of its segment when it starts, and announces that it has finished by adding 1 to the
// bits above kLenBits of lens[b,l].  The workgroup that finds all others of the segment already
// counted stores the new plain length, which also clears the count.  Between launches lens holds plain
// lengths (< 2^20).
#include "pkv_common.hpp"

namespace pkv {

constexpr int kLenBits = 20;
constexpr int kLenMask = (1 << kLenBits) - 1;

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
};

// Cache rows are read once per decode step and never reused by the same launch: stream them past the
// caches (nontemporal) so that they do not evict each other on the way in.
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;
__device__ __forceinline__ uint4 load_stream16(const unsigned char* p) {
    const u32x4_t t = __builtin_nontemporal_load((const u32x4_t*)p);
    return make_uint4(t.x, t.y, t.z, t.w);
}

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

// One sub-block of SB = NI * (64/LPR) rows starting at row r0 of the segment, for the G query heads of
// the group: online-softmax update of (mrun, srun, o).  LPR lanes cover one row with 16 bytes each.
// TAIL = false: every row is an occupied cache slot.  TAIL = true: rows >= len are masked, and the row
// len_old, if it is being appended (app), comes from k_new/v_new and is written to its slot (writer).
template <bool BF16, int LPR, int G, int NI, bool TAIL>
__device__ __forceinline__ void attend_block(const unsigned char* __restrict__ kseg,
                                             const unsigned char* __restrict__ vseg, int r0, int len,
                                             int len_old, bool app, bool writer,
                                             const unsigned char* __restrict__ knew,
                                             const unsigned char* __restrict__ vnew, unsigned char* kw,
                                             unsigned char* vw, int row_bytes, int sub, int rg,
                                             const float (&qf)[G][BF16 ? 8 : 4], float (&o)[G][BF16 ? 8 : 4],
                                             float (&mrun)[G], float (&srun)[G]) {
    constexpr int EPL = BF16 ? 8 : 4;
    constexpr int RPI = kWave / LPR;
    uint4 kr[NI], vr[NI];
    const uint32_t lane_off = (uint32_t)(r0 + rg) * (uint32_t)row_bytes + (uint32_t)sub * 16u;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const uint32_t o_i = lane_off + (uint32_t)(i * RPI) * (uint32_t)row_bytes;
        if constexpr (!TAIL) {
            kr[i] = load_stream16(kseg + o_i);
            vr[i] = load_stream16(vseg + o_i);
        } else {
            const int r = r0 + i * RPI + rg;
            kr[i] = make_uint4(0, 0, 0, 0); vr[i] = make_uint4(0, 0, 0, 0);
            if (r < len) {
                const bool isnew = app && r == len_old;
                kr[i] = load_stream16(isnew ? knew + sub * 16 : kseg + o_i);
                vr[i] = load_stream16(isnew ? vnew + sub * 16 : vseg + o_i);
                if (isnew && writer) {
                    *(uint4*)(kw + o_i) = kr[i];
                    *(uint4*)(vw + o_i) = vr[i];
                }
            }
        }
    }
    float s[G][NI], mx[G];
#pragma unroll
    for (int g = 0; g < G; ++g) mx[g] = -INFINITY;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        float kf[EPL];
        unpack16<BF16>(kr[i], kf);
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float d = 0.f;
#pragma unroll
            for (int x = 0; x < EPL; ++x) d = fmaf(qf[g][x], kf[x], d);
#pragma unroll
            for (int sh = 1; sh < LPR; sh <<= 1) d += __shfl_xor(d, sh, kWave);
            if constexpr (TAIL) d = (r0 + i * RPI + rg < len) ? d : -INFINITY;
            s[g][i] = d;
            mx[g] = fmaxf(mx[g], d);
        }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
        for (int sh = LPR; sh < kWave; sh <<= 1) mx[g] = fmaxf(mx[g], __shfl_xor(mx[g], sh, kWave));
        // the caller guarantees r0 < len: some row is valid, so mx is finite
        const float mnew = fmaxf(mrun[g], mx[g]);
        const float corr = __builtin_amdgcn_exp2f(mrun[g] - mnew);  // 0 on the first block
        mrun[g] = mnew;
        srun[g] *= corr;
#pragma unroll
        for (int x = 0; x < EPL; ++x) o[g][x] *= corr;
    }
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        float vf[EPL];
        unpack16<BF16>(vr[i], vf);
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float pr = __builtin_amdgcn_exp2f(s[g][i] - mrun[g]);
            srun[g] += pr;   // per row group; the groups are merged at the end
#pragma unroll
            for (int x = 0; x < EPL; ++x) o[g][x] = fmaf(pr, vf[x], o[g][x]);
        }
    }
}

// W wavefronts per workgroup; OCC = wavefronts per SIMD the register allocation must allow.
template <bool BF16, int LPR, int G, int NI, int W, int OCC>
__global__ void __launch_bounds__(W * kWave, OCC)
decode_attn_kernel(DecodeParams p) {
    constexpr int EPL = BF16 ? 8 : 4;            // elements per lane (16 bytes)
    constexpr int RPI = kWave / LPR;             // rows per wavefront-wide load instruction
    constexpr int SB = NI * RPI;                 // rows per sub-block
    constexpr int NSB = kDecodeChunk / SB;       // sub-blocks per chunk
    constexpr int ESZ = BF16 ? 2 : 4;
    constexpr int DMAX = 128;
    static_assert(kDecodeChunk % SB == 0 && NSB >= 1, "chunk must be a whole number of sub-blocks");
    __shared__ float s_part[W][G][DMAX + 2];

    const int HU = p.H / G;                      // workgroups (head groups) per segment
    const int hu = blockIdx.x % HU, i_seg = blockIdx.x / HU;
    const int b = i_seg / p.nl, l = p.l0 + i_seg % p.nl, sl = b * p.L + l;
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave;
    const int sub = lane % LPR, rg = lane / LPR;
    const int row_bytes = p.D * ESZ;

    const int len_old = __hip_atomic_load(p.lens + sl, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & kLenMask;
    const int cap = p.caps[sl];
    const int64_t off = p.seg_off[sl];
    const bool app = p.append && len_old < cap;
    const int len = len_old + (app ? 1 : 0);
    const int nch = (len + kDecodeChunk - 1) / kDecodeChunk;
    const int kvh = (hu * G) / p.grp;
    const bool writer = app && ((hu * G) % p.grp == 0);
    const int64_t segbase = (off * p.Hkv + (int64_t)kvh * cap) * row_bytes;
    const int64_t newrow = ((int64_t)sl * p.Hkv + kvh) * row_bytes;

    float o[G][EPL], mrun[G], srun[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        mrun[g] = -INFINITY; srun[g] = 0.f;
#pragma unroll
        for (int x = 0; x < EPL; ++x) o[g][x] = 0.f;
    }

    if (wv < nch) {
        float qf[G][EPL];
        const float qs = p.scale[l] * 1.4426950408889634f;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const uint4 qr = *(const uint4*)(p.q + ((int64_t)sl * p.H + hu * G + g) * row_bytes + sub * 16);
            unpack16<BF16>(qr, qf[g]);
#pragma unroll
            for (int x = 0; x < EPL; ++x) qf[g][x] *= qs;
        }
        const unsigned char* kseg = p.kc + segbase;
        const unsigned char* vseg = p.vc + segbase;
        for (int c = wv; c < nch; c += W) {
            const bool full = (c + 1) * kDecodeChunk <= len_old;   // no masked row, no appended row
#pragma unroll
            for (int sb = 0; sb < NSB; ++sb) {
                const int r0 = c * kDecodeChunk + sb * SB;
                if (full) {
                    attend_block<BF16, LPR, G, NI, false>(kseg, vseg, r0, len, len_old, app, writer, nullptr, nullptr,
                                                          nullptr, nullptr, row_bytes, sub, rg, qf, o, mrun, srun);
                } else if (r0 < len) {
                    attend_block<BF16, LPR, G, NI, true>(kseg, vseg, r0, len, len_old, app, writer,
                                                         p.k_new + newrow, p.v_new + newrow, p.kc + segbase,
                                                         p.vc + segbase, row_bytes, sub, rg, qf, o, mrun, srun);
                }
            }
        }
        // merge the RPI row groups of the wavefront (they share mrun)
#pragma unroll
        for (int g = 0; g < G; ++g) {
#pragma unroll
            for (int sh = LPR; sh < kWave; sh <<= 1) {
                srun[g] += __shfl_xor(srun[g], sh, kWave);
#pragma unroll
                for (int x = 0; x < EPL; ++x) o[g][x] += __shfl_xor(o[g][x], sh, kWave);
            }
        }
    }
    if (rg == 0) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float* dst = s_part[wv][g];
#pragma unroll
            for (int x = 0; x < EPL; ++x) dst[sub * EPL + x] = o[g][x];
            if (sub == 0) { dst[DMAX] = mrun[g]; dst[DMAX + 1] = srun[g]; }
        }
    }
    __syncthreads();
    // merge the wavefronts: thread (g, d)
    for (int i = threadIdx.x; i < G * p.D; i += blockDim.x) {
        const int g = i / p.D, d = i % p.D;
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < W; ++w) M = fmaxf(M, s_part[w][g][DMAX]);
        float num = 0.f, den = 0.f;
        if (M > -INFINITY) {
#pragma unroll
            for (int w = 0; w < W; ++w) {
                const float wgt = __builtin_amdgcn_exp2f(s_part[w][g][DMAX] - M);
                num = fmaf(wgt, s_part[w][g][d], num);
                den = fmaf(wgt, s_part[w][g][DMAX + 1], den);
            }
        }
        const float r = den > 0.f ? num / den : 0.f;   // an empty segment gives zeros
        const size_t oi = ((size_t)sl * p.H + hu * G + g) * p.D + d;
        if constexpr (BF16) ((bf16_t*)p.out)[oi] = f32_to_bf16(r); else ((float*)p.out)[oi] = r;
    }
    // every thread of this workgroup has read lens (before the barrier); count the workgroup in
    if (threadIdx.x == 0) {
        const int old = atomicAdd(p.lens + sl, 1 << kLenBits);
        if ((int)((unsigned)old >> kLenBits) == HU - 1)
            __hip_atomic_store(p.lens + sl, len, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

size_t decode_ws_bytes(const pkv_shape&) { return 0; }

static int pick_group(int grp) { return grp % 8 == 0 ? 8 : grp % 4 == 0 ? 4 : grp % 2 == 0 ? 2 : 1; }

// Launch shapes.  All workgroups of a launch should be resident at once (one round), so short
// segments get small workgroups with many row loads in flight per wavefront, and long segments get
// more wavefronts per workgroup to shorten the serial walk over the chunks:
//   shape 0: 2 wavefronts, 16 loads in flight, 2 wavefronts/SIMD   (segments up to ~1k tokens)
//   shape 1: 4 wavefronts,  8 loads in flight, 4 wavefronts/SIMD   (up to ~4k tokens)
//   shape 2: 8 wavefronts,  8 loads in flight, 4 wavefronts/SIMD   (longer)
// Groups of 4 or 8 query heads keep 8 loads in flight and 2 wavefronts/SIMD (register budget).
template <bool BF16, int LPR, int G>
static hipError_t launch_decode_s(const DecodeParams& p, int shape, int nblk, hipStream_t st) {
    constexpr int RPI = kWave / LPR;
    constexpr int NI_MAX = kDecodeChunk / RPI;
    constexpr bool WIDE = G >= 4;
    constexpr int NI16 = WIDE ? (NI_MAX < 8 ? NI_MAX : 8) : (NI_MAX < 16 ? NI_MAX : 16);
    constexpr int NI8 = NI_MAX < 8 ? NI_MAX : 8;
    constexpr int OCC4 = WIDE ? 2 : 4;
    if (shape == 0)
        hipLaunchKernelGGL((decode_attn_kernel<BF16, LPR, G, NI16, 2, 2>), dim3(nblk), dim3(2 * kWave), 0, st, p);
    else if (shape == 1)
        hipLaunchKernelGGL((decode_attn_kernel<BF16, LPR, G, NI8, 4, OCC4>), dim3(nblk), dim3(4 * kWave), 0, st, p);
    else
        hipLaunchKernelGGL((decode_attn_kernel<BF16, LPR, G, NI8, 8, OCC4>), dim3(nblk), dim3(8 * kWave), 0, st, p);
    return hipGetLastError();
}

template <bool BF16, int LPR>
static hipError_t launch_decode_g(const DecodeParams& p, int G, int shape, int nblk, hipStream_t st) {
    switch (G) {
        case 8: return launch_decode_s<BF16, LPR, 8>(p, shape, nblk, st);
        case 4: return launch_decode_s<BF16, LPR, 4>(p, shape, nblk, st);
        case 2: return launch_decode_s<BF16, LPR, 2>(p, shape, nblk, st);
        default: return launch_decode_s<BF16, LPR, 1>(p, shape, nblk, st);
    }
}

hipError_t launch_decode(const pkv_shape& s, int l0, int l1, const void* q, const void* k_new,
                         const void* v_new, const float* scale, void* kc, void* vc,
                         const int64_t* seg_off, const int32_t* caps, int32_t* lens, void* out,
                         hipStream_t st) {
    DecodeParams p;
    p.B = s.B; p.L = s.L; p.l0 = l0; p.nl = l1 - l0; p.H = s.H; p.Hkv = s.Hkv; p.D = s.D;
    p.grp = s.H / s.Hkv; p.append = k_new != nullptr;
    p.q = (const unsigned char*)q; p.k_new = (const unsigned char*)k_new;
    p.v_new = (const unsigned char*)v_new; p.scale = scale;
    p.kc = (unsigned char*)kc; p.vc = (unsigned char*)vc; p.seg_off = seg_off; p.caps = caps;
    p.lens = lens; p.out = (unsigned char*)out;
    const int G = pick_group(p.grp);
    const int nblk = s.B * p.nl * (s.H / G);
    const bool bf16 = s.dtype == PKV_BF16;
    const int lpr = s.D * (bf16 ? 2 : 4) / 16;
    const int shape = s.N <= 1024 ? 0 : s.N <= 4096 ? 1 : 2;   // segments hold at most N + appended tokens
    if (bf16) {
        if (lpr == 8) return launch_decode_g<true, 8>(p, G, shape, nblk, st);
        return launch_decode_g<true, 16>(p, G, shape, nblk, st);
    }
    if (lpr == 16) return launch_decode_g<false, 16>(p, G, shape, nblk, st);
    return launch_decode_g<false, 32>(p, G, shape, nblk, st);
}

}  // namespace pkv
