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
    // pruning at a fixed distance (decode_attn_kernel<..., EV = true> only)
    int N, t, d;                  // prompt length, 1-based decode step, distance
    const int32_t* base_lens;     // [B,L] entries kept after prefill
    int32_t* kept_pos;            // one int per slot, may be null
};

// Virtual row numbering of a segment under pruning: rows [0, perm) are the permanent slots, rows
// perm + j are ring slot j (the last d+1 slots of the segment).  r_new is the row of the token stored
// in this step, r_mask the row of a token pruned in this step (-1 if none).
struct RingMap {
    int shift;    // ring slot j is physical slot perm + j + shift
    int r_new;
    int r_mask;
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
template <bool BF16, int LPR, int G, int NI, bool TAIL, bool EV = false>
__device__ __forceinline__ void attend_block(const unsigned char* __restrict__ kseg,
                                             const unsigned char* __restrict__ vseg, int r0, int len,
                                             int len_old, bool app, bool writer, const RingMap& ring,
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
            if constexpr (!EV) {
                if (r < len) {
                    const bool isnew = app && r == len_old;
                    kr[i] = load_stream16(isnew ? knew + sub * 16 : kseg + o_i);
                    vr[i] = load_stream16(isnew ? vnew + sub * 16 : vseg + o_i);
                    if (isnew && writer) {
                        *(uint4*)(kw + o_i) = kr[i];
                        *(uint4*)(vw + o_i) = vr[i];
                    }
                }
            } else {
                if (r < len && r != ring.r_mask) {
                    const uint32_t o_s = o_i + (r >= len_old ? (uint32_t)ring.shift * (uint32_t)row_bytes : 0u);
                    const bool isnew = r == ring.r_new;
                    kr[i] = load_stream16(isnew ? knew + sub * 16 : kseg + o_s);
                    vr[i] = load_stream16(isnew ? vnew + sub * 16 : vseg + o_s);
                    if (isnew && writer) {
                        *(uint4*)(kw + o_s) = kr[i];
                        *(uint4*)(vw + o_s) = vr[i];
                    }
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
            if constexpr (TAIL) {
                const int r = r0 + i * RPI + rg;
                d = (r < len && (!EV || r != ring.r_mask)) ? d : -INFINITY;
            }
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
template <bool BF16, int LPR, int G, int NI, int W, int OCC, bool EV = false>
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
    // plain step: append at slot len_old.  Pruning step: len_old counts the permanent entries, the new
    // token goes to ring slot (t-1) mod (d+1), and the token stored d steps ago (ring slot t mod (d+1))
    // either becomes permanent entry len_old or is left out from now on.
    bool app = p.append && len_old < cap;
    int len = len_old + (app ? 1 : 0), len_next = len;
    RingMap ring = {0, -1, -1};
    int ring0 = 0, cs = 0;
    bool grad = false, decide = false;
    if constexpr (EV) {
        const int base = p.base_lens[sl];
        ring0 = cap - (p.d + 1);
        app = base >= 0 && ring0 >= base && len_old <= ring0;   // else: capacity cannot hold the ring
        decide = app && p.t > p.d;
        cs = p.t % (p.d + 1);
        long long target = (2ll * base * ((long long)p.N + p.t) + p.N) / (2ll * p.N);
        target = target < 1 ? 1 : target;
        grad = decide && (long long)len_old + p.d + 1 <= target && len_old < ring0;
        ring.shift = ring0 - len_old;
        ring.r_new = len_old + (p.t - 1) % (p.d + 1);
        ring.r_mask = (decide && !grad) ? len_old + cs : -1;
        len = app ? len_old + (p.t < p.d + 1 ? p.t : p.d + 1) : 0;
        len_next = len_old + (grad ? 1 : 0);
    }
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
                    attend_block<BF16, LPR, G, NI, false>(kseg, vseg, r0, len, len_old, app, writer, ring, nullptr,
                                                          nullptr, nullptr, nullptr, row_bytes, sub, rg, qf, o,
                                                          mrun, srun);
                } else if (r0 < len) {
                    if constexpr (EV) {   // a sub-block whose only occupied row is the pruned one has no work
                        const int hi = len < r0 + SB ? len : r0 + SB;
                        if (hi - r0 == 1 && ring.r_mask == r0) continue;
                    }
                    attend_block<BF16, LPR, G, NI, true, EV>(kseg, vseg, r0, len, len_old, app, writer, ring,
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
    if constexpr (EV) {
        // the surviving token moves from its ring slot to the next permanent slot.  Attention above read it
        // from the ring slot; nobody reads the permanent slot in this launch.
        if (grad && writer && wv == 0 && rg == 0) {
            const unsigned char* src_k = p.kc + segbase + (size_t)(ring0 + cs) * row_bytes + sub * 16;
            const unsigned char* src_v = p.vc + segbase + (size_t)(ring0 + cs) * row_bytes + sub * 16;
            *(uint4*)(p.kc + segbase + (size_t)len_old * row_bytes + sub * 16) = *(const uint4*)src_k;
            *(uint4*)(p.vc + segbase + (size_t)len_old * row_bytes + sub * 16) = *(const uint4*)src_v;
        }
        if (p.kept_pos && app && hu == 0 && threadIdx.x == 0) {
            int32_t* kp = p.kept_pos + off;
            kp[ring0 + (p.t - 1) % (p.d + 1)] = p.N + p.t - 1;
            if (decide) {
                if (grad) kp[len_old] = p.N + p.t - p.d - 1;
                kp[ring0 + cs] = -1;
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
            __hip_atomic_store(p.lens + sl, len_next, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

size_t decode_ws_bytes(const pkv_shape&) { return 0; }

static int pick_group(int grp) { return grp % 8 == 0 ? 8 : grp % 4 == 0 ? 4 : grp % 2 == 0 ? 2 : 1; }

// Launch shapes.  All workgroups of a launch should be resident at once (one round), so short
// segments get small workgroups with many row loads in flight per wavefront, and long segments get
// more wavefronts per workgroup to shorten the serial walk over the chunks:
//   shape 0: 2 wavefronts, 16 loads in flight, 2 wavefronts/SIMD   (segments up to ~1k tokens);
//            with more than one resident round of workgroups: 4 loads in flight, 4 wavefronts/SIMD
//   shape 1: 4 wavefronts,  8 loads in flight, 4 wavefronts/SIMD   (up to ~4k tokens)
//   shape 2: 8 wavefronts,  8 loads in flight, 4 wavefronts/SIMD   (longer)
// Groups of 4 or 8 query heads keep 8 loads in flight and 2 wavefronts/SIMD (register budget).
// Number of compute units of the current device (queried once per device).
static int compute_units() {
    static int cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) n = 256;
        cached[dev] = n;
    }
    return cached[dev];
}

template <bool BF16, int LPR, int G, bool EV>
static hipError_t launch_decode_s(const DecodeParams& p, int shape, int nblk, hipStream_t st) {
    constexpr int RPI = kWave / LPR;
    constexpr int NI_MAX = kDecodeChunk / RPI;
    constexpr bool WIDE = G >= 4;
    constexpr int NI16 = WIDE ? (NI_MAX < 8 ? NI_MAX : 8) : (NI_MAX < 16 ? NI_MAX : 16);
    constexpr int NI8 = NI_MAX < 8 ? NI_MAX : 8;
    constexpr int OCC4 = WIDE ? 2 : 4;
    if constexpr (!WIDE) {
        // more workgroups than fit on the chip at once: smaller register footprint, twice as many resident
        // workgroups with a quarter of the loads in flight each (measured 4-27 % faster from batch 2 on)
        constexpr int NI4 = NI_MAX < 4 ? NI_MAX : 4;
        if (shape == 0 && nblk > 4 * compute_units()) {
            hipLaunchKernelGGL((decode_attn_kernel<BF16, LPR, G, NI4, 2, 4, EV>), dim3(nblk), dim3(2 * kWave), 0, st, p);
            return hipGetLastError();
        }
    }
    if (shape == 0)
        hipLaunchKernelGGL((decode_attn_kernel<BF16, LPR, G, NI16, 2, 2, EV>), dim3(nblk), dim3(2 * kWave), 0, st, p);
    else if (shape == 1)
        hipLaunchKernelGGL((decode_attn_kernel<BF16, LPR, G, NI8, 4, OCC4, EV>), dim3(nblk), dim3(4 * kWave), 0, st, p);
    else
        hipLaunchKernelGGL((decode_attn_kernel<BF16, LPR, G, NI8, 8, OCC4, EV>), dim3(nblk), dim3(8 * kWave), 0, st, p);
    return hipGetLastError();
}

template <bool BF16, int LPR, bool EV>
static hipError_t launch_decode_g(const DecodeParams& p, int G, int shape, int nblk, hipStream_t st) {
    switch (G) {
        case 8: return launch_decode_s<BF16, LPR, 8, EV>(p, shape, nblk, st);
        case 4: return launch_decode_s<BF16, LPR, 4, EV>(p, shape, nblk, st);
        case 2: return launch_decode_s<BF16, LPR, 2, EV>(p, shape, nblk, st);
        default: return launch_decode_s<BF16, LPR, 1, EV>(p, shape, nblk, st);
    }
}

template <bool EV>
static hipError_t launch_decode_any(const pkv_shape& s, const DecodeParams& p, hipStream_t st) {
    const int G = pick_group(p.grp);
    const int nblk = s.B * p.nl * (s.H / G);
    const bool bf16 = s.dtype == PKV_BF16;
    const int lpr = s.D * (bf16 ? 2 : 4) / 16;
    const int shape = s.N <= 1024 ? 0 : s.N <= 4096 ? 1 : 2;   // segments hold at most N + appended tokens
    if (bf16) {
        if (lpr == 8) return launch_decode_g<true, 8, EV>(p, G, shape, nblk, st);
        return launch_decode_g<true, 16, EV>(p, G, shape, nblk, st);
    }
    if (lpr == 16) return launch_decode_g<false, 16, EV>(p, G, shape, nblk, st);
    return launch_decode_g<false, 32, EV>(p, G, shape, nblk, st);
}

static DecodeParams make_params(const pkv_shape& s, int l0, int l1, const void* q, const void* k_new,
                                const void* v_new, const float* scale, void* kc, void* vc,
                                const int64_t* seg_off, const int32_t* caps, int32_t* lens, void* out) {
    DecodeParams p;
    p.B = s.B; p.L = s.L; p.l0 = l0; p.nl = l1 - l0; p.H = s.H; p.Hkv = s.Hkv; p.D = s.D;
    p.grp = s.H / s.Hkv; p.append = k_new != nullptr;
    p.q = (const unsigned char*)q; p.k_new = (const unsigned char*)k_new;
    p.v_new = (const unsigned char*)v_new; p.scale = scale;
    p.kc = (unsigned char*)kc; p.vc = (unsigned char*)vc; p.seg_off = seg_off; p.caps = caps;
    p.lens = lens; p.out = (unsigned char*)out;
    p.N = s.N; p.t = 0; p.d = 0; p.base_lens = nullptr; p.kept_pos = nullptr;
    return p;
}

hipError_t launch_decode(const pkv_shape& s, int l0, int l1, const void* q, const void* k_new,
                         const void* v_new, const float* scale, void* kc, void* vc,
                         const int64_t* seg_off, const int32_t* caps, int32_t* lens, void* out,
                         hipStream_t st) {
    const DecodeParams p = make_params(s, l0, l1, q, k_new, v_new, scale, kc, vc, seg_off, caps, lens, out);
    return launch_decode_any<false>(s, p, st);
}

hipError_t launch_decode_evict(const pkv_shape& s, int l0, int l1, const void* q, const void* k_new,
                               const void* v_new, const float* scale, void* kc, void* vc,
                               const int64_t* seg_off, const int32_t* caps, const int32_t* base_lens,
                               int32_t* lens, int32_t* kept_pos, int t, int d, void* out, hipStream_t st) {
    DecodeParams p = make_params(s, l0, l1, q, k_new, v_new, scale, kc, vc, seg_off, caps, lens, out);
    p.t = t; p.d = d; p.base_lens = base_lens; p.kept_pos = kept_pos;
    return launch_decode_any<true>(s, p, st);
}

}  // namespace pkv
