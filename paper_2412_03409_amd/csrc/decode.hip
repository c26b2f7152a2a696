// Stage 4b: one decode step over the ragged compressed cache (Sec. 3.1: the newest token's query
// interacts with the cached KV vectors of every layer).  ONE kernel per step (two for bf16 caches whose
// KV heads serve several query heads: a planning kernel and decode_gqa_kernel, further down):
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

static int pick_group(int grp) { return grp % 8 == 0 ? 8 : grp % 4 == 0 ? 4 : grp % 2 == 0 ? 2 : 1; }

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
    // work list of the grouped-query kernel (see decode_plan_kernel)
    int G, n_seg, S0, pieces_cap, record_word, partial_word;
    int* plan;
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

// ---------------------------------------------------------------------------------------------------
// Grouped-query variant on the matrix cores (bf16 storage, G = 2, 4 or 8 query heads per KV head).
// With several query heads per cached row the dot products dominate the vector ALU, so they move to
// MFMA: scores^T[16 rows x 16 head columns] = K[16 rows x D] . Q^T[D x heads] with
// v_mfma_f32_16x16x32_bf16 (A = cache rows, one row per lane%16, 8 consecutive bf16 per lane; B = the
// queries, head lane%16, columns >= G are zero).  A lane then holds the scores of one head for 4 rows;
// softmax runs in that layout (one exp per (row, head) instead of one per lane of the row), the
// probabilities go through a per-wavefront LDS tile to the layout of the V rows (LPR lanes per row, as in
// the kernel above), and the weighted V sum stays on the vector ALU with fp32 accumulators.
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

// Partial results cross workgroups (and XCDs) inside one launch: device-scope relaxed atomics go straight
// to the coherent level and need no cache-wide write-back or invalidate.
__device__ __forceinline__ void st_agent(float* p, float v) {
    __hip_atomic_store((unsigned*)p, __float_as_uint(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_agent(const float* p) {
    return __uint_as_float(__hip_atomic_load((const unsigned*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}

__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// State of one segment for this step, computed identically by every workgroup that touches it.
struct SegState {
    int len_old;   // occupied slots before the step (under pruning: permanent entries)
    int cap;
    int len;       // rows to attend to in this step (virtual rows under pruning)
    int len_next;  // value of lens after the step
    int ring0, cs; // pruning: first ring slot, ring slot of the token decided in this step
    bool app, grad, decide;
    RingMap ring;
    int64_t off;
};

template <bool EV>
__device__ __forceinline__ SegState seg_state(const DecodeParams& p, int sl) {
    SegState s;
    s.len_old = __hip_atomic_load(p.lens + sl, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & kLenMask;
    s.cap = p.caps[sl];
    s.off = p.seg_off[sl];
    s.app = p.append && s.len_old < s.cap;
    s.len = s.len_old + (s.app ? 1 : 0);
    s.len_next = s.len;
    s.ring = {0, s.app ? s.len_old : -1, -1};
    s.ring0 = 0; s.cs = 0; s.grad = false; s.decide = false;
    if constexpr (EV) {
        const int base = p.base_lens[sl];
        s.ring0 = s.cap - (p.d + 1);
        s.app = base >= 0 && s.ring0 >= base && s.len_old <= s.ring0;
        s.decide = s.app && p.t > p.d;
        s.cs = p.t % (p.d + 1);
        long long target = (2ll * base * ((long long)p.N + p.t) + p.N) / (2ll * p.N);
        target = target < 1 ? 1 : target;
        s.grad = s.decide && (long long)s.len_old + p.d + 1 <= target && s.len_old < s.ring0;
        s.ring.shift = s.ring0 - s.len_old;
        s.ring.r_new = s.app ? s.len_old + (p.t - 1) % (p.d + 1) : -1;
        s.ring.r_mask = (s.decide && !s.grad) ? s.len_old + s.cs : -1;
        s.len = s.app ? s.len_old + (p.t < p.d + 1 ? p.t : p.d + 1) : 0;
        s.len_next = s.len_old + (s.grad ? 1 : 0);
    }
    return s;
}

// Work list for the grouped-query kernel.  PrefixKV gives the layers very different lengths (tens of rows
// next to thousands), so a segment is cut into pieces of S rows and every (piece, head group) is one
// work item of similar size.  The planning kernel (one workgroup) evaluates the state of every segment
// once, writes one 64-byte record per piece with everything the attention kernel needs, and advances
// lens itself, so the attention kernel neither reads nor counts on lens.
// Layout of the workspace, in 32-bit words:
//   [0] next item to claim  [1] number of items  [2] S  [3] number of pieces  [4] number of full pieces
//   [16 ...]  arrive[n_seg * HU], records[pieces_cap][16] (64-byte aligned),
//   then the partial results of split segments: [pieces_cap * HU][G][D + 2] floats.
// S starts at S0 and doubles until the pieces fit the table.
constexpr int kPlanThreads = 1024;
constexpr int kPlanHdr = 16;
constexpr int kRecWords = 16;
enum { REC_SL = 0, REC_SPLIT, REC_NSPLIT, REC_FIRST, REC_LEN_OLD, REC_LEN, REC_CAP, REC_FLAGS, REC_OFF_LO,
       REC_OFF_HI, REC_SHIFT, REC_RNEW, REC_RMASK, REC_RING0, REC_CS, REC_LAST };
enum { RECF_APP = 1, RECF_GRAD = 2, RECF_DECIDE = 4 };

constexpr int kPlanClasses = 16;
// Size class of a segment's last piece: 0 for the longest remainders.
__device__ __forceinline__ int last_piece_class(int len, int S) {
    int np = (len + S - 1) / S;
    np = np < 1 ? 1 : np;
    const int rows = len - (np - 1) * S;                 // 0 .. S
    const int c = (int)(((long long)rows * kPlanClasses) / ((long long)S + 1));   // 0 .. kPlanClasses-1
    return kPlanClasses - 1 - c;
}

// sum over the workgroup and exclusive prefix of v (blockDim.x a multiple of 64, at most 1024): wavefront
// shuffles and one pass over the wavefront totals
__device__ __forceinline__ int plan_scan(int v, int* s_wave, int& total) {
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave, nw = blockDim.x / kWave;
    int incl = v;
    for (int d = 1; d < kWave; d <<= 1) {
        const int up = __shfl_up(incl, d, kWave);
        if (lane >= d) incl += up;
    }
    __syncthreads();                         // s_wave may still be read from the previous call
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

template <bool EV>
__global__ void __launch_bounds__(kPlanThreads)
decode_plan_kernel(DecodeParams p) {
    __shared__ int s_wave[kPlanThreads / kWave];
    __shared__ int s_cls[kPlanClasses];
    const int tid = threadIdx.x, n = p.n_seg;
    const int nt = blockDim.x;               // a power of two, 64 .. kPlanThreads: no more wavefronts than the segments need
    const int per = (n + nt - 1) / nt;
    const int lo = tid * per < n ? tid * per : n, hi = lo + per < n ? lo + per : n;
    int* hdr = p.plan;
    int* arrive = p.plan + kPlanHdr;
    int* records = p.plan + p.record_word;
    auto seg_of = [&](int i) { return (i / p.nl) * p.L + p.l0 + i % p.nl; };
    // Up to kPlanThreads segments (the usual case) are one per thread: its state is read once and kept.
    const bool single = per == 1;
    SegState mine_ss;
    if (single && lo < hi) mine_ss = seg_state<EV>(p, seg_of(lo));
    auto state = [&](int i) { return single ? mine_ss : seg_state<EV>(p, seg_of(i)); };
    if (tid < kPlanClasses) s_cls[tid] = 0;
    // Items are claimed from a counter in list order, so the list holds the full pieces first and the last
    // (shorter) piece of every segment at the end: the tail of the launch is made of small items.
    int S = p.S0, total_full = 0, mine = 0, at = 0;
    for (;;) {
        mine = 0;
        for (int i = lo; i < hi; ++i) {
            const int len = state(i).len;
            const int np = (len + S - 1) / S;
            mine += np < 1 ? 0 : np - 1;      // full pieces; every segment has exactly one last piece
        }
        at = plan_scan(mine, s_wave, total_full);
        if (total_full + n <= p.pieces_cap || S >= (1 << 24)) break;
        S *= 2;
    }
    const int total = total_full + n;
    const bool ok = total <= p.pieces_cap;   // cannot fail for pieces_cap >= n_seg
    // the last pieces go into the list by size class, largest first (the order inside a class is arbitrary;
    // results do not depend on the order of the list); s_cls was cleared before the barriers of the scan
    for (int i = lo; i < hi; ++i) atomicAdd(&s_cls[last_piece_class(state(i).len, S)], 1);
    __syncthreads();
    if (tid == 0) {
        int run = 0;
        for (int c = 0; c < kPlanClasses; ++c) { const int v = s_cls[c]; s_cls[c] = run; run += v; }
    }
    __syncthreads();
    if (ok) {
        for (int i = lo; i < hi; ++i) {
            const int sl = seg_of(i);
            const SegState ss = state(i);
            int np = (ss.len + S - 1) / S;
            np = np < 1 ? 1 : np;
            const int last = total_full + atomicAdd(&s_cls[last_piece_class(ss.len, S)], 1);
            for (int k = 0; k < np; ++k) {
                int* r = records + (size_t)(k < np - 1 ? at + k : last) * kRecWords;
                r[REC_SL] = sl; r[REC_SPLIT] = k; r[REC_NSPLIT] = np; r[REC_FIRST] = at;
                r[REC_LEN_OLD] = ss.len_old; r[REC_LEN] = ss.len; r[REC_CAP] = ss.cap;
                r[REC_FLAGS] = (ss.app ? RECF_APP : 0) | (ss.grad ? RECF_GRAD : 0) | (ss.decide ? RECF_DECIDE : 0);
                r[REC_OFF_LO] = (int)(uint32_t)ss.off; r[REC_OFF_HI] = (int)(ss.off >> 32);
                r[REC_SHIFT] = ss.ring.shift; r[REC_RNEW] = ss.ring.r_new; r[REC_RMASK] = ss.ring.r_mask;
                r[REC_RING0] = ss.ring0; r[REC_CS] = ss.cs; r[REC_LAST] = last;
            }
            at += np - 1;
            p.lens[sl] = ss.len_next;        // the records carry the old state; nobody else reads lens in this step
        }
    }
    const int HU = p.H / p.G;
    for (int i = tid; i < n * HU; i += nt) arrive[i] = 0;
    if (tid == 0) { hdr[0] = 0; hdr[1] = ok ? total * HU : 0; hdr[2] = S; hdr[3] = ok ? total : 0; hdr[4] = total_full; }
}

// Persistent kernel: as many workgroups as fit on the chip; a workgroup starts with the item of its own
// index and claims further items of the list from a counter.
template <int D, int G, int NT, int W, int OCC, bool EV>
__global__ void __launch_bounds__(W * kWave, OCC)
decode_gqa_kernel(DecodeParams p) {
    constexpr int LPR = D / 8;                   // lanes per V row (16 bytes each)
    constexpr int RPI = kWave / LPR;             // V rows per wavefront-wide load
    constexpr int NJ = D / 32;                   // MFMAs per 16-row tile
    constexpr int BR = NT * 16;                  // rows per block
    constexpr int VI = BR / RPI;                 // V loads per block
    constexpr int GP = G < 4 ? 4 : G;            // head columns kept in LDS
    constexpr int DMAX = 128;
    constexpr int ROWB = D * 2;
    constexpr int PST = D + 2;                   // floats per (item, head) partial: numerators, max, denominator
    static_assert(D == 64 || D == 128, "head dimension");
    __shared__ float s_part[2][W][G][DMAX + 2];   // double-buffered across items: no barrier at the end of an item
    __shared__ __attribute__((aligned(16))) float s_p[W][BR * GP];
    __shared__ __attribute__((aligned(16))) float s_corr[W][GP];
    __shared__ int s_last[2];
    __shared__ int s_next[2];

    const int HU = p.H / G;
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave;
    const int sub = lane % LPR, rg = lane / LPR;     // V layout
    const int kr = lane & 15, kq = lane >> 4;        // K / score layout: row (or head) kr, quad kq
    int* hdr = p.plan;
    int* arrive = p.plan + kPlanHdr;
    const int* records = p.plan + p.record_word;
    float* partial = (float*)(p.plan + p.partial_word);
    const int total = hdr[1], S = hdr[2];

  // every workgroup starts with the item of its own index and claims further ones from a counter; the claim
  // for the next item is issued first, so its round trip is hidden behind the work on this one
  for (int item = blockIdx.x, it = 0; item < total; ++it) {
    if (threadIdx.x == 0) s_next[it & 1] = atomicAdd(hdr, 1) + (int)gridDim.x;
    const int piece = item / HU, hu = item % HU;
    const int* rec = records + (size_t)piece * kRecWords;
    const int sl = rec[REC_SL], split = rec[REC_SPLIT], nsplit = rec[REC_NSPLIT], first_full = rec[REC_FIRST];
    const int len_old = rec[REC_LEN_OLD], len = rec[REC_LEN], cap = rec[REC_CAP], flags = rec[REC_FLAGS];
    const int64_t seg_tok = (int64_t)(((uint64_t)(uint32_t)rec[REC_OFF_HI] << 32) | (uint32_t)rec[REC_OFF_LO]);
    const RingMap ring = {rec[REC_SHIFT], rec[REC_RNEW], rec[REC_RMASK]};
    const int l = sl % p.L;
    const int row_lo = split * S;
    const int row_hi = len < row_lo + S ? len : row_lo + S;
    const int nblk = row_hi > row_lo ? (row_hi - row_lo + BR - 1) / BR : 0;
    const int kvh = (hu * G) / p.grp;
    const bool writer = (flags & RECF_APP) && ((hu * G) % p.grp == 0);
    const int64_t segbase = (seg_tok * p.Hkv + (int64_t)kvh * cap) * ROWB;
    const unsigned char* knew = p.k_new + ((int64_t)sl * p.Hkv + kvh) * ROWB;
    const unsigned char* vnew = p.v_new + ((int64_t)sl * p.Hkv + kvh) * ROWB;
    unsigned char* kseg = p.kc + segbase;
    unsigned char* vseg = p.vc + segbase;
    float (*spart)[G][DMAX + 2] = s_part[it & 1];

    float o[G][8], m_run = -INFINITY, l_run = 0.f;
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int x = 0; x < 8; ++x) o[g][x] = 0.f;

    if (wv < nblk) {
        const float qs = p.scale[l] * 1.4426950408889634f;
        bf16x8_t qb[NJ];
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            uint4 t = make_uint4(0, 0, 0, 0);
            if (kr < G) t = *(const uint4*)(p.q + ((int64_t)sl * p.H + hu * G + kr) * ROWB + (4 * j + kq) * 16);
            qb[j] = __builtin_bit_cast(bf16x8_t, t);
        }
        float* ps = s_p[wv];
        float* cr = s_corr[wv];
        for (int blk = wv; blk < nblk; blk += W) {
            const int r0 = row_lo + blk * BR;
            const bool full = r0 + BR <= len_old;
            if constexpr (EV) {
                const int hi = len < r0 + BR ? len : r0 + BR;
                if (hi - r0 == 1 && ring.r_mask == r0) continue;
            }
            uint4 kf[NT][NJ], vr[VI];
            if (full) {
#pragma unroll
                for (int t = 0; t < NT; ++t)
#pragma unroll
                    for (int j = 0; j < NJ; ++j)
                        kf[t][j] = load_stream16(kseg + (uint32_t)(r0 + 16 * t + kr) * ROWB + (4 * j + kq) * 16);
#pragma unroll
                for (int i = 0; i < VI; ++i)
                    vr[i] = load_stream16(vseg + (uint32_t)(r0 + i * RPI + rg) * ROWB + sub * 16);
            } else {
                // guarded path: rows past the end are zero, the new row comes from k_new / v_new and is stored,
                // under pruning ring rows map to the ring slots and the pruned row is left out
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    const int r = r0 + 16 * t + kr;
                    const bool valid = r < len && r != ring.r_mask;
                    const bool isnew = r == ring.r_new;
                    const uint32_t so = (uint32_t)(r + ((EV && r >= len_old) ? ring.shift : 0)) * ROWB;
#pragma unroll
                    for (int j = 0; j < NJ; ++j) {
                        const int c16 = (4 * j + kq) * 16;
                        kf[t][j] = make_uint4(0, 0, 0, 0);
                        if (valid) {
                            kf[t][j] = load_stream16(isnew ? knew + c16 : kseg + so + c16);
                            if (isnew && writer) *(uint4*)(kseg + so + c16) = kf[t][j];
                        }
                    }
                }
#pragma unroll
                for (int i = 0; i < VI; ++i) {
                    const int r = r0 + i * RPI + rg;
                    const bool valid = r < len && r != ring.r_mask;
                    const bool isnew = r == ring.r_new;
                    const uint32_t so = (uint32_t)(r + ((EV && r >= len_old) ? ring.shift : 0)) * ROWB;
                    vr[i] = make_uint4(0, 0, 0, 0);
                    if (valid) {
                        vr[i] = load_stream16(isnew ? vnew + sub * 16 : vseg + so + sub * 16);
                        if (isnew && writer) *(uint4*)(vseg + so + sub * 16) = vr[i];
                    }
                }
            }
            // scores: one MFMA chain per 16-row tile
            f32x4_t acc[NT];
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                acc[t] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int j = 0; j < NJ; ++j)
                    acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kf[t][j]), qb[j],
                                                                     acc[t], 0, 0, 0);
            }
            float mx = -INFINITY;
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float sc = acc[t][r] * qs;
                    if (!full) {
                        const int row = r0 + 16 * t + 4 * kq + r;
                        sc = (row < len && row != ring.r_mask) ? sc : -INFINITY;
                    }
                    acc[t][r] = sc;
                    mx = fmaxf(mx, sc);
                }
            mx = fmaxf(mx, __shfl_xor(mx, 16, kWave));
            mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
            const float mnew = fmaxf(m_run, mx);              // finite: the block has an occupied row
            const float corr = __builtin_amdgcn_exp2f(m_run - mnew);
            m_run = mnew;
            float psum = 0.f;
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float pr = __builtin_amdgcn_exp2f(acc[t][r] - mnew);
                    psum += pr;
                    if (kr < GP) ps[(16 * t + 4 * kq + r) * GP + kr] = pr;
                }
            l_run = l_run * corr + psum;
            if (kq == 0 && kr < GP) cr[kr] = corr;
            wave_lds_sync();
            float cg[GP];
#pragma unroll
            for (int g4 = 0; g4 < GP; g4 += 4) {
                const float4 c4 = *(const float4*)(cr + g4);
                cg[g4] = c4.x; cg[g4 + 1] = c4.y; cg[g4 + 2] = c4.z; cg[g4 + 3] = c4.w;
            }
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int x = 0; x < 8; ++x) o[g][x] *= cg[g];
#pragma unroll
            for (int i = 0; i < VI; ++i) {
                float vf[8], pg[GP];
                unpack16<true>(vr[i], vf);
#pragma unroll
                for (int g4 = 0; g4 < GP; g4 += 4) {
                    const float4 p4 = *(const float4*)(ps + (i * RPI + rg) * GP + g4);
                    pg[g4] = p4.x; pg[g4 + 1] = p4.y; pg[g4 + 2] = p4.z; pg[g4 + 3] = p4.w;
                }
#pragma unroll
                for (int g = 0; g < G; ++g)
#pragma unroll
                    for (int x = 0; x < 8; ++x) o[g][x] = fmaf(pg[g], vf[x], o[g][x]);
            }
            wave_lds_sync();
        }
        // the four quads hold partial row sums of the same head; the RPI row groups partial outputs
        l_run += __shfl_xor(l_run, 16, kWave);
        l_run += __shfl_xor(l_run, 32, kWave);
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int sh = LPR; sh < kWave; sh <<= 1)
#pragma unroll
                for (int x = 0; x < 8; ++x) o[g][x] += __shfl_xor(o[g][x], sh, kWave);
    }
    if constexpr (EV) {
        if (split == 0) {
            const int ring0 = rec[REC_RING0], cs = rec[REC_CS];
            if ((flags & RECF_GRAD) && writer && wv == 0 && rg == 0) {
                const size_t src = (size_t)(ring0 + cs) * ROWB + sub * 16, dst = (size_t)len_old * ROWB + sub * 16;
                *(uint4*)(kseg + dst) = *(const uint4*)(kseg + src);
                *(uint4*)(vseg + dst) = *(const uint4*)(vseg + src);
            }
            if (p.kept_pos && (flags & RECF_APP) && hu == 0 && threadIdx.x == 0) {
                int32_t* kp = p.kept_pos + seg_tok;
                kp[ring0 + (p.t - 1) % (p.d + 1)] = p.N + p.t - 1;
                if (flags & RECF_DECIDE) {
                    if (flags & RECF_GRAD) kp[len_old] = p.N + p.t - p.d - 1;
                    kp[ring0 + cs] = -1;
                }
            }
        }
    }
    if (rg == 0) {
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int x = 0; x < 8; ++x) spart[wv][g][sub * 8 + x] = o[g][x];
    }
    if (kq == 0 && kr < G) { spart[wv][kr][DMAX] = m_run; spart[wv][kr][DMAX + 1] = l_run; }
    __syncthreads();
    const int item_next = __builtin_amdgcn_readfirstlane(s_next[it & 1]);   // uniform, stays in scalar registers
    // merge the wavefronts: thread (g, d).  A whole segment is written out; a piece leaves (numerators,
    // max, denominator) in the workspace and the last piece of the (segment, head group) to arrive adds them up
    float* mine = partial + ((size_t)piece * HU + hu) * (G * PST);
    for (int i = threadIdx.x; i < G * D; i += blockDim.x) {
        const int g = i / D, d = i % D;
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < W; ++w) M = fmaxf(M, spart[w][g][DMAX]);
        float num = 0.f, den = 0.f;
        if (M > -INFINITY) {
#pragma unroll
            for (int w = 0; w < W; ++w) {
                const float wgt = __builtin_amdgcn_exp2f(spart[w][g][DMAX] - M);
                num = fmaf(wgt, spart[w][g][d], num);
                den = fmaf(wgt, spart[w][g][DMAX + 1], den);
            }
        }
        if (nsplit == 1) {
            const float r = den > 0.f ? num / den : 0.f;   // an empty segment gives zeros
            ((bf16_t*)p.out)[((size_t)sl * p.H + hu * G + g) * D + d] = f32_to_bf16(r);
        } else {
            st_agent(mine + g * PST + d, num);
            if (d == 0) { st_agent(mine + g * PST + D, M); st_agent(mine + g * PST + D + 1, den); }
        }
    }
    if (nsplit > 1) {
        // Hand-off of the partial to the last arriver.  Every thread waits until its own partial stores have
        // been acknowledged (they are device-scope write-through stores, so acknowledged = at the level all
        // XCDs share), the barrier collects the workgroup, then one thread counts the workgroup in.
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
        __syncthreads();
        const int i_seg = (sl / p.L) * p.nl + (sl % p.L - p.l0);
#ifdef PKV_GQA_RELEASE_ACQUIRE
        // the same hand-off inside the HIP memory model: release on the arrival, acquire in the last arriver
        if (threadIdx.x == 0)
            s_last[it & 1] = __hip_atomic_fetch_add(arrive + i_seg * HU + hu, 1, __ATOMIC_ACQ_REL,
                                                    __HIP_MEMORY_SCOPE_AGENT) == nsplit - 1;
#else
        if (threadIdx.x == 0) s_last[it & 1] = atomicAdd(arrive + i_seg * HU + hu, 1) == nsplit - 1;
#endif
        __syncthreads();
        if (s_last[it & 1]) {
            // the partial of piece k sits at the piece's place in the list
            const int last_piece = rec[REC_LAST];
            for (int i = threadIdx.x; i < G * D; i += blockDim.x) {
                const int g = i / D, d = i % D;
                float M = -INFINITY;
                for (int k = 0; k < nsplit; ++k) {
                    const int pc = k < nsplit - 1 ? first_full + k : last_piece;
                    M = fmaxf(M, ld_agent(partial + ((size_t)pc * HU + hu) * (G * PST) + g * PST + D));
                }
                float num = 0.f, den = 0.f;
                if (M > -INFINITY) {
                    for (int k = 0; k < nsplit; ++k) {
                        const int pc = k < nsplit - 1 ? first_full + k : last_piece;
                        const float* pk = partial + ((size_t)pc * HU + hu) * (G * PST) + g * PST;
                        const float wgt = __builtin_amdgcn_exp2f(ld_agent(pk + D) - M);
                        num = fmaf(wgt, ld_agent(pk + d), num);
                        den = fmaf(wgt, ld_agent(pk + D + 1), den);
                    }
                }
                const float r = den > 0.f ? num / den : 0.f;
                ((bf16_t*)p.out)[((size_t)sl * p.H + hu * G + g) * D + d] = f32_to_bf16(r);
            }
        }
    }
    item = item_next;
  }
}



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
    constexpr int OCC4 = WIDE ? 2 : 3;   // the 4- and 8-wavefront shapes spill at 4 wavefronts/SIMD (8-9 % slower)
    if constexpr (!WIDE) {
        // more workgroups than fit on the chip at once: smaller register footprint, twice as many resident
        // workgroups with a quarter of the loads in flight each (measured 4-27 % faster from batch 2 on)
        constexpr int NI4 = NI_MAX < 4 ? NI_MAX : 4;
        const bool one_round = nblk <= 4 * compute_units();
        // bf16 rows: the two-wavefront shapes also serve longer prompts (measured at N = 1500 .. 8192: 4-18 %
        // faster than four or eight wavefronts per workgroup, whose register budget spills) except when
        // segments of more than 4096 rows meet a launch of several rounds
        if (BF16 && (shape == 1 || (shape == 2 && one_round))) shape = 0;
        if (shape == 0 && !one_round) {
            // the pruning variant needs more registers: at 4 wavefronts/SIMD it spills (measured 10-22 % slower)
            constexpr int OCC_MANY = EV ? 3 : 4;
            hipLaunchKernelGGL((decode_attn_kernel<BF16, LPR, G, NI4, 2, OCC_MANY, EV>), dim3(nblk), dim3(2 * kWave), 0, st, p);
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
    if constexpr (!BF16) {   // bf16 caches with several query heads per KV head use decode_gqa_kernel instead
        switch (G) {
            case 8: return launch_decode_s<BF16, LPR, 8, EV>(p, shape, nblk, st);
            case 4: return launch_decode_s<BF16, LPR, 4, EV>(p, shape, nblk, st);
            case 2: return launch_decode_s<BF16, LPR, 2, EV>(p, shape, nblk, st);
            default: break;
        }
    }
    return launch_decode_s<BF16, LPR, 1, EV>(p, shape, nblk, st);
}

// Workspace layout of the grouped-query path for n_seg segments (see decode_plan_kernel).
struct GqaLayout {
    int pieces_cap, record_word, partial_word;
    size_t bytes;
};
static GqaLayout gqa_layout(int n_seg, int H, int G, int D, int N) {
    GqaLayout g;
    const int HU = H / G;
    g.pieces_cap = n_seg * (2 + N / 512);
    g.record_word = (int)(((size_t)kPlanHdr + (size_t)n_seg * HU + 15) / 16 * 16);
    g.partial_word = g.record_word + g.pieces_cap * kRecWords;
    g.bytes = ((size_t)g.partial_word + (size_t)g.pieces_cap * HU * G * (D + 2)) * 4;
    return g;
}

size_t decode_ws_bytes(const pkv_shape& s) {
    const int G = pick_group(s.H / s.Hkv);
    if (s.dtype != PKV_BF16 || G < 2) return 0;
    return gqa_layout(s.B * s.L, s.H, G, s.D, s.N).bytes;
}

// Grouped-query bf16 launches: the planning kernel, then one resident round of workgroups of W wavefronts
// (2 wavefronts per SIMD) that claim (piece, head group) items until the list is empty.
template <int D, int G, bool EV>
static hipError_t launch_gqa_s(DecodeParams p, const pkv_shape& s, int* ws, hipStream_t st) {
    constexpr int W = 4;
    // Only the 4-wavefront workgroup is instantiated.  8-wavefront workgroups (with 2048-row pieces) were slower
    // on every workload they were measured on, and one run of that shape ended in a GPU fault whose cause is
    // not known; the shape must not be used until it is.
    static_assert(W == 4, "decode_gqa_kernel is validated for 4 wavefronts per workgroup only");
    const GqaLayout lay = gqa_layout(s.B * p.nl, s.H, G, D, s.N);
    p.G = G; p.n_seg = s.B * p.nl; p.S0 = 1024; p.pieces_cap = lay.pieces_cap; p.record_word = lay.record_word; p.partial_word = lay.partial_word;
    p.plan = ws;
    int plan_threads = kWave;
    while (plan_threads < p.n_seg && plan_threads < kPlanThreads) plan_threads <<= 1;
    hipLaunchKernelGGL((decode_plan_kernel<EV>), dim3(1), dim3(plan_threads), 0, st, p);
    int grid = compute_units() * (8 / W);
    const long long most = (long long)lay.pieces_cap * (s.H / G);
    if (grid > most) grid = (int)most;
    // 32-row blocks: with 64-row blocks the eight-head kernel spills at D = 128 (54.1 vs 50.7 us per step) and
    // the four-head kernel sits at the register limit (124.2 vs 119.9 us per step on the long-context workload)
    constexpr int NT = 2;
    hipLaunchKernelGGL((decode_gqa_kernel<D, G, NT, W, 2, EV>), dim3(grid), dim3(W * kWave), 0, st, p);
    return hipGetLastError();
}

template <int D, bool EV>
static hipError_t launch_gqa(const DecodeParams& p, const pkv_shape& s, int G, int* ws, hipStream_t st) {
    switch (G) {
        case 8: return launch_gqa_s<D, 8, EV>(p, s, ws, st);
        case 4: return launch_gqa_s<D, 4, EV>(p, s, ws, st);
        default: return launch_gqa_s<D, 2, EV>(p, s, ws, st);
    }
}

template <bool EV>
static hipError_t launch_decode_any(const pkv_shape& s, const DecodeParams& p, void* ws, hipStream_t st) {
    const int G = pick_group(p.grp);
    const int nblk = s.B * p.nl * (s.H / G);
    const bool bf16 = s.dtype == PKV_BF16;
    if (bf16 && G >= 2)     // several query heads share the cached rows: scores on the matrix cores
        return s.D == 128 ? launch_gqa<128, EV>(p, s, G, (int*)ws, st) : launch_gqa<64, EV>(p, s, G, (int*)ws, st);
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
    p.G = 1; p.n_seg = 0; p.S0 = 0; p.pieces_cap = 0; p.record_word = 0; p.partial_word = 0; p.plan = nullptr;
    return p;
}

hipError_t launch_decode(const pkv_shape& s, int l0, int l1, const void* q, const void* k_new,
                         const void* v_new, const float* scale, void* kc, void* vc,
                         const int64_t* seg_off, const int32_t* caps, int32_t* lens, void* out, void* ws,
                         hipStream_t st) {
    const DecodeParams p = make_params(s, l0, l1, q, k_new, v_new, scale, kc, vc, seg_off, caps, lens, out);
    return launch_decode_any<false>(s, p, ws, st);
}

hipError_t launch_decode_evict(const pkv_shape& s, int l0, int l1, const void* q, const void* k_new,
                               const void* v_new, const float* scale, void* kc, void* vc,
                               const int64_t* seg_off, const int32_t* caps, const int32_t* base_lens,
                               int32_t* lens, int32_t* kept_pos, int t, int d, void* out, void* ws,
                               hipStream_t st) {
    DecodeParams p = make_params(s, l0, l1, q, k_new, v_new, scale, kc, vc, seg_off, caps, lens, out);
    p.t = t; p.d = d; p.base_lens = base_lens; p.kept_pos = kept_pos;
    return launch_decode_any<true>(s, p, ws, st);
}

}  // namespace pkv
