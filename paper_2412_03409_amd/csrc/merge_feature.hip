// Cache merging by feature similarity (Sec. 4.3, "Eviction or merging", the variant called "Feature"):
// every pruned vector is averaged into the retained vector of the same head it is most similar to,
// matching metric = cosine.  Keys are matched by key similarity and values by value similarity (the paper
// describes the operation on keys and applies "the same" to values), every head on its own.
//
//  mf_prepare_kernel   per (tensor, segment, kv head): marks the retained positions in the assignment row
//                      (-1) and computes 1/|x_u| of every retained vector.
//  mf_match_kernel     one workgroup = 256 positions of one (tensor, segment, kv head), a wavefront owns 64
//                      (two 32-position tiles, so that a fragment read from LDS feeds two MFMAs).
//                      The retained vectors (already contiguous in the compacted cache) stream through LDS
//                      64 at a time (asynchronous copies, double-buffered) and
//                        S^T[32 slots x 32 positions] = Xc[32 x D] . X^T
//                      runs on v_mfma_f32_32x32x16_bf16.  In the accumulator layout a lane holds one position
//                      and 16 slots in ascending order, so the running (best score, slot) pair is per lane
//                      and the two halves of a column meet once at the end.  |x_m| is a positive factor
//                      common to all candidates of position m and is left out; score = dot * 1/|x_u|.
//  mf_average_kernel   per (tensor, segment, kv head): sorts the pruned positions by (slot, position) in LDS, so
//                      that the members of a slot are one run; a wavefront sums the rows of a run, 64/LPR rows
//                      per load and four loads deep, in a fixed order (fp32), then stores the mean.
#include "pkv_common.hpp"

namespace pkv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

constexpr int kMfTiles = 2;     // 32-position tiles per wavefront of the matching kernel: a fragment read feeds that many MFMAs
constexpr int kMfRows = 128 * kMfTiles;   // positions per workgroup of the matching kernel
constexpr int kMfStage = 64;    // retained vectors per LDS stage

struct MergeFeatureParams {
    int L, Hkv, N, NP;          // NP = N rounded up to 64: pitch of the norm rows
    int U, nmb;                 // (segment, kv head) pairs; 128-position blocks per pair
    const bf16_t* x[2]; Strides xs[2];
    bf16_t* xc[2];
    const int64_t* seg_off; const int32_t* caps; const int32_t* kept_pos; const int32_t* lens;
    int32_t* match;             // [2][B*L*Hkv][N]
    float* inv_norm;            // [2][B*L*Hkv][NP]
    int np2;                    // N rounded up to a power of two (>= 64): keys sorted by the averaging kernel
};

// chunk swizzle of the staged rows (16-byte chunk c of row r sits at c ^ swz(r)): the fragment reads touch
// 32 consecutive rows at one chunk
template <int CPR>
__device__ __forceinline__ int mf_swz(int r) {
    if constexpr (CPR == 16) return ((r & 3) << 2) | ((r >> 2) & 3);
    else return ((r & 1) << 2) | ((r >> 1) & 3);
}

template <int LPR>
__global__ void __launch_bounds__(256)
mf_prepare_kernel(MergeFeatureParams p) {
    constexpr int RPI = kWave / LPR;
    __shared__ int32_t skp[kMaxN];
    const int u = blockIdx.x % p.U, tz = blockIdx.x / p.U;
    const int seg = u / p.Hkv, h = u % p.Hkv;
    const int n = min(p.lens[seg], p.N);
    const int64_t off = p.seg_off[seg];
    const int cap = p.caps[seg];
    for (int j = threadIdx.x; j < n; j += blockDim.x) skp[j] = p.kept_pos[off + j];
    __syncthreads();
    // retained positions: binary search in the ascending list
    int32_t* mrow = p.match + ((size_t)tz * p.U + u) * p.N;
    for (int m = threadIdx.x; m < p.N; m += blockDim.x) {
        int lo = 0, hi = n;               // first slot with kept_pos >= m
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (skp[mid] < m) lo = mid + 1; else hi = mid;
        }
        mrow[m] = (lo < n && skp[lo] == m) ? -1 : 0;
    }
    // reciprocal norms of the retained vectors, 0 for a zero vector; zero fill up to the pitch
    float* nrow = p.inv_norm + ((size_t)tz * p.U + u) * p.NP;
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave;
    const int sub = lane % LPR, rg = lane / LPR;
    const bf16_t* base = p.xc[tz] + ((size_t)off * p.Hkv + (size_t)h * cap) * (LPR * 8);
    for (int j0 = wv * RPI; j0 < n; j0 += 4 * RPI) {
        const int j = j0 + rg;
        float ss = 0.f;
        if (j < n) {
            const uint4 w4 = *(const uint4*)(base + (size_t)j * (LPR * 8) + sub * 8);
            const uint32_t w[4] = {w4.x, w4.y, w4.z, w4.w};
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                const float a = __uint_as_float(w[x] << 16), b = __uint_as_float(w[x] & 0xffff0000u);
                ss = fmaf(a, a, ss);
                ss = fmaf(b, b, ss);
            }
        }
#pragma unroll
        for (int sh = 1; sh < LPR; sh <<= 1) ss += __shfl_xor(ss, sh, kWave);
        if (j < n && sub == 0) nrow[j] = ss > 0.f ? 1.0f / sqrtf(ss) : 0.f;
    }
    for (int j = n + threadIdx.x; j < p.NP; j += blockDim.x) nrow[j] = 0.f;
}

template <int D>
__global__ void __launch_bounds__(256, 2)
mf_match_kernel(MergeFeatureParams p) {
    constexpr int ROWB = D * 2;
    constexpr int CPR = D / 8;
    constexpr int NJ = D / 16;
    __shared__ __attribute__((aligned(1024))) unsigned char sXa[kMfStage * ROWB];
    __shared__ __attribute__((aligned(1024))) unsigned char sXb[kMfStage * ROWB];
    __shared__ __attribute__((aligned(256))) float sNa[kMfStage];
    __shared__ __attribute__((aligned(256))) float sNb[kMfStage];

    const int U = p.U;
    const int u = (blockIdx.x / p.nmb) % U, tz = blockIdx.x / (p.nmb * U);
    const int seg = u / p.Hkv, h = u % p.Hkv;
    const int n = p.lens[seg];
    const int m0 = (blockIdx.x % p.nmb) * kMfRows;
    if (n >= p.N || n < 1) return;               // nothing was pruned
    const int b = seg / p.L, l = seg % p.L;
    const Strides xs = p.xs[tz];
    const bf16_t* xbase = p.x[tz] + xs.b * b + xs.l * l + xs.h * h;
    const bf16_t* cbase = p.xc[tz] + ((size_t)p.seg_off[seg] * p.Hkv + (size_t)h * p.caps[seg]) * D;
    const float* nrow = p.inv_norm + ((size_t)tz * U + u) * p.NP;
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave;
    const int ln = lane & 31, hf = lane >> 5;
    constexpr int T = kMfTiles;
    int pos_m[T];                                // the positions this lane's columns belong to
    bf16x8_t qf[T][NJ];
#pragma unroll
    for (int t = 0; t < T; ++t) {
        pos_m[t] = m0 + (wv * T + t) * 32 + ln;
        const int row = pos_m[t] < p.N ? pos_m[t] : p.N - 1;
#pragma unroll
        for (int j = 0; j < NJ; ++j)
            qf[t][j] = __builtin_bit_cast(bf16x8_t, *(const uint4*)(xbase + (uint32_t)row * (uint32_t)xs.n + 16 * j + 8 * hf));
    }
    const int nst = (n + kMfStage - 1) / kMfStage;

    constexpr int kInst = kMfStage * ROWB / 1024 / 4;    // 16-byte copy instructions per wavefront
    int cp_row[kInst], cp_col[kInst];
#pragma unroll
    for (int i = 0; i < kInst; ++i) {
        const int idx = (wv * kInst + i) * 64 + lane;
        const int r = idx / CPR, pos = idx % CPR;
        cp_row[i] = r;
        cp_col[i] = 8 * (pos ^ mf_swz<CPR>(r));
    }
    auto issue = [&](int st, unsigned char* dX, float* dN) {
#pragma unroll
        for (int i = 0; i < kInst; ++i) {
            int row = st * kMfStage + cp_row[i];
            row = row < n ? row : n - 1;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(cbase + ((uint32_t)row * (uint32_t)D + (uint32_t)cp_col[i])),
                                             (__attribute__((address_space(3))) void*)(dX + (wv * kInst + i) * 1024), 16, 0, 0);
        }
        if (wv == 0)   // the 64 reciprocal norms of the stage (the row is padded to a multiple of 64)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(nrow + st * kMfStage + lane),
                                             (__attribute__((address_space(3))) void*)dN, 4, 0, 0);
    };

    float best[T];
    int bslot[T];
#pragma unroll
    for (int t = 0; t < T; ++t) { best[t] = -INFINITY; bslot[t] = 0; }
    auto step = [&](int st, const unsigned char* sX, const float* sN, unsigned char* nX, float* nN) {
        __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0): this wavefront's copies of stage st have landed
        __syncthreads();
        if (st + 1 < nst) issue(st + 1, nX, nN);
#pragma unroll
        for (int half = 0; half < kMfStage / 32; ++half) {
            const int slot0 = st * kMfStage + half * 32;
            if (slot0 >= n) break;
            const unsigned char* sK = sX + half * 32 * ROWB;
            f32x16_t s[T];
#pragma unroll
            for (int t = 0; t < T; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) s[t][r] = 0.f;
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                const int pos = (2 * j + hf) ^ mf_swz<CPR>(ln);
                const bf16x8_t kf = __builtin_bit_cast(bf16x8_t, *(const uint4*)(sK + ln * ROWB + pos * 16));
#pragma unroll
                for (int t = 0; t < T; ++t) s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[t][j], s[t], 0, 0, 0);
            }
            // register r holds slot slot0 + 8*(r/4) + 4*hf + r%4: ascending in r
            const bool tail = slot0 + 32 > n;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const float4 iv = *(const float4*)(sN + half * 32 + 8 * g + 4 * hf);
                const float inv[4] = {iv.x, iv.y, iv.z, iv.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int slot = slot0 + 8 * g + 4 * hf + e;
#pragma unroll
                    for (int t = 0; t < T; ++t) {
                        float sc = s[t][4 * g + e] * inv[e];
                        if (tail) sc = slot < n ? sc : -INFINITY;
                        const bool up = sc > best[t];   // strict: the first maximum stays
                        best[t] = up ? sc : best[t];
                        bslot[t] = up ? slot : bslot[t];
                    }
                }
            }
        }
    };

    issue(0, sXa, sNa);
    for (int st = 0; st < nst; st += 2) {
        step(st, sXa, sNa, sXb, sNb);
        if (st + 1 < nst) step(st + 1, sXb, sNb, sXa, sNa);
    }
    // the two halves of a column: larger score, on a tie the lower slot
    int32_t* mrow = p.match + ((size_t)tz * U + u) * p.N;
#pragma unroll
    for (int t = 0; t < T; ++t) {
        const float ob = __shfl_xor(best[t], 32, kWave);
        const int os = __shfl_xor(bslot[t], 32, kWave);
        if (ob > best[t] || (ob == best[t] && os < bslot[t])) { best[t] = ob; bslot[t] = os; }
        if (hf == 0 && pos_m[t] < p.N && mrow[pos_m[t]] != -1) mrow[pos_m[t]] = bslot[t];
    }
}

// 8 bf16 of a row added to fp32 sums; the mean of 8 sums stored as bf16 (round to nearest even)
__device__ __forceinline__ void add_row(float (&acc)[8], const uint4& w4) {
    const uint32_t w[4] = {w4.x, w4.y, w4.z, w4.w};
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        acc[2 * x] += __uint_as_float(w[x] << 16);
        acc[2 * x + 1] += __uint_as_float(w[x] & 0xffff0000u);
    }
}
__device__ __forceinline__ void store_mean(bf16_t* dst, const float (&acc)[8], float cnt) {
    uint32_t o[4];
#pragma unroll
    for (int x = 0; x < 4; ++x)
        o[x] = (uint32_t)f32_to_bf16(acc[2 * x] / cnt) | ((uint32_t)f32_to_bf16(acc[2 * x + 1] / cnt) << 16);
    *(uint4*)dst = make_uint4(o[0], o[1], o[2], o[3]);
}

// One workgroup per (tensor, segment, kv head).  The pruned positions are sorted by (slot, position) -- keys
// slot << 13 | position, retained positions as the largest key, a bitonic network in LDS -- so that the members
// of every slot are one contiguous, ascending run.  A wavefront then takes 64 slots at a time (each lane finds
// the run of one slot by binary search); a row group (LPR lanes, 16 bytes of the row each) sums the run of one
// slot in ascending order, four loads deep; a run longer than kLongRun is summed by all row groups of the
// wavefront together, in a fixed order.
template <int LPR>
__global__ void __launch_bounds__(1024)
mf_average_kernel(MergeFeatureParams p) {
    constexpr int RPI = kWave / LPR;             // rows per wavefront-wide load
    constexpr int kDeep = 4;                     // loads in flight per row group
    constexpr int kLongRun = 64;
    extern __shared__ __attribute__((aligned(16))) uint32_t keys[];   // np2 keys
    const int U = p.U;
    const int u = blockIdx.x % U, tz = blockIdx.x / U;
    const int seg = u / p.Hkv, h = u % p.Hkv;
    const int n = p.lens[seg];
    if (n >= p.N || n < 1) return;               // nothing was pruned: the compacted rows stay as they are
    const int b = seg / p.L, l = seg % p.L;
    const int64_t off = p.seg_off[seg];
    const int32_t* kp = p.kept_pos + off;
    const Strides xs = p.xs[tz];
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave, nwv = blockDim.x / kWave;
    const int sub = lane % LPR, rg = lane / LPR;
    const bf16_t* xbase = p.x[tz] + xs.b * b + xs.l * l + xs.h * h + sub * 8;
    bf16_t* cbase = p.xc[tz] + ((size_t)off * p.Hkv + (size_t)h * p.caps[seg]) * (LPR * 8) + sub * 8;
    const int32_t* mrow = p.match + ((size_t)tz * U + u) * p.N;
    const int np2 = p.np2;
    for (int m = threadIdx.x; m < np2; m += blockDim.x) {
        const int slot = m < p.N ? mrow[m] : -1;
        keys[m] = (slot >= 0 && slot < n) ? ((uint32_t)slot << 13) | (uint32_t)m : 0xffffffffu;
    }
    __syncthreads();
    for (int k = 2; k <= np2; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int t = threadIdx.x; t < np2 / 2; t += blockDim.x) {
                const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1)), q = i | j;
                const uint32_t a = keys[i], c = keys[q];
                if ((a > c) == ((i & k) == 0)) { keys[i] = c; keys[q] = a; }
            }
            // the 64 pairs a wavefront takes per turn of a stage with partner distance j <= 64 lie in one aligned
            // block of 128 keys, the same for all such stages: only a stage that reaches further (or is followed
            // by one that does) has to meet the other wavefronts
            const int jn = j > 1 ? (j >> 1) : k;
            if (j > kWave || jn > kWave) {
                __syncthreads();
            } else {
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            }
        }

    // slots per wavefront and turn: up to 64, fewer when that leaves wavefronts without work
    const int bs = min(kWave, ((n + nwv - 1) / nwv + RPI - 1) / RPI * RPI);
    for (int jb = wv * bs; jb < n; jb += nwv * bs) {
        // lane s: the run of slot jb + s = [first key >= slot << 13, first key >= (slot + 1) << 13)
        int lo_l, hi_l;
        {
            const uint32_t t0 = (uint32_t)(jb + lane) << 13, t1 = t0 + (1u << 13);
            int lo = 0, hi = np2;
            while (lo < hi) { const int mid = (lo + hi) >> 1; if (keys[mid] < t0) lo = mid + 1; else hi = mid; }
            lo_l = lo;
            hi = np2;
            while (lo < hi) { const int mid = (lo + hi) >> 1; if (keys[mid] < t1) lo = mid + 1; else hi = mid; }
            hi_l = lo;
        }
        const int ns = min(bs, n - jb);
        const unsigned long long longmask = __builtin_amdgcn_ballot_w64(lane < ns && hi_l - lo_l > kLongRun);
        // runs of ordinary length: one row group per slot, RPI slots of the wavefront at a time
        for (int s0 = 0; s0 < ns; s0 += RPI) {
            const int s = s0 + rg;               // < 64
            const bool act = s < ns && !((longmask >> s) & 1ull);
            // (both shuffles outside any condition: a lane that sits out must still serve as a source)
            const int lo = __shfl(lo_l, s, kWave), hi_s = __shfl(hi_l, s, kWave);
            const int hi = act ? hi_s : lo;
            float acc[8];
#pragma unroll
            for (int x = 0; x < 8; ++x) acc[x] = 0.f;
            uint4 own = make_uint4(0, 0, 0, 0);  // zero bits are 0.0
            if (act) own = *(const uint4*)(xbase + (uint32_t)kp[jb + s] * (uint32_t)xs.n);   // the retained vector
            for (int i0 = lo; i0 < hi; i0 += kDeep) {
                uint4 r[kDeep];
#pragma unroll
                for (int d = 0; d < kDeep; ++d) {
                    r[d] = make_uint4(0, 0, 0, 0);
                    if (i0 + d < hi) r[d] = *(const uint4*)(xbase + (keys[i0 + d] & 8191u) * (uint32_t)xs.n);
                }
#pragma unroll
                for (int d = 0; d < kDeep; ++d) add_row(acc, r[d]);
            }
            add_row(acc, own);
            if (act) store_mean(cbase + (size_t)(jb + s) * (LPR * 8), acc, (float)(hi - lo + 1));
        }
        // long runs (few retained vectors, or one that attracts everything): the whole wavefront per slot
        for (unsigned long long lm = longmask; lm; lm &= lm - 1) {
            const int s = __builtin_ctzll(lm);
            const int lo = __shfl(lo_l, s, kWave), hi = __shfl(hi_l, s, kWave);
            float acc[8];
#pragma unroll
            for (int x = 0; x < 8; ++x) acc[x] = 0.f;
            uint4 own = make_uint4(0, 0, 0, 0);
            if (rg == 0) own = *(const uint4*)(xbase + (uint32_t)kp[jb + s] * (uint32_t)xs.n);
            for (int i0 = lo; i0 < hi; i0 += kDeep * RPI) {
                uint4 r[kDeep];
#pragma unroll
                for (int d = 0; d < kDeep; ++d) {
                    const int i = i0 + d * RPI + rg;
                    r[d] = make_uint4(0, 0, 0, 0);
                    if (i < hi) r[d] = *(const uint4*)(xbase + (keys[i] & 8191u) * (uint32_t)xs.n);
                }
#pragma unroll
                for (int d = 0; d < kDeep; ++d) add_row(acc, r[d]);
            }
            add_row(acc, own);
#pragma unroll
            for (int sh = LPR; sh < kWave; sh <<= 1)
#pragma unroll
                for (int x = 0; x < 8; ++x) acc[x] += __shfl_xor(acc[x], sh, kWave);
            if (rg == 0) store_mean(cbase + (size_t)(jb + s) * (LPR * 8), acc, (float)(hi - lo + 1));
        }
    }
}

size_t merge_feature_ws_bytes(const pkv_shape& s) {
    const size_t np = ((size_t)s.N + 63) & ~(size_t)63;
    return 2 * (size_t)s.B * s.L * s.Hkv * np * sizeof(float);
}

hipError_t launch_merge_feature(const pkv_shape& s, const void* k, Strides ks, const void* v, Strides vs,
                                const int64_t* seg_off, const int32_t* caps, const int32_t* kept_pos,
                                const int32_t* lens, void* kc, void* vc, int32_t* match, void* ws,
                                hipStream_t st) {
    MergeFeatureParams p;
    p.L = s.L; p.Hkv = s.Hkv; p.N = s.N; p.NP = (s.N + 63) & ~63;
    p.x[0] = (const bf16_t*)k; p.x[1] = (const bf16_t*)v; p.xs[0] = ks; p.xs[1] = vs;
    p.xc[0] = (bf16_t*)kc; p.xc[1] = (bf16_t*)vc;
    p.seg_off = seg_off; p.caps = caps; p.kept_pos = kept_pos; p.lens = lens;
    p.match = match; p.inv_norm = (float*)ws;
    const int U = s.B * s.L * s.Hkv;
    p.U = U;
    int np2 = 64;
    while (np2 < s.N) np2 <<= 1;
    p.np2 = np2;
    const int nt = np2 <= 2048 ? 256 : 1024;
    const size_t lds = (size_t)np2 * sizeof(uint32_t);
    p.nmb = (s.N + kMfRows - 1) / kMfRows;
    const dim3 g_prep(2u * U), g_match(2u * U * p.nmb), g_avg(2u * U);
    if (s.D == 128) {
        hipLaunchKernelGGL(mf_prepare_kernel<16>, g_prep, dim3(256), 0, st, p);
        hipLaunchKernelGGL(mf_match_kernel<128>, g_match, dim3(256), 0, st, p);
        hipLaunchKernelGGL(mf_average_kernel<16>, g_avg, dim3(nt), lds, st, p);
    } else {
        hipLaunchKernelGGL(mf_prepare_kernel<8>, g_prep, dim3(256), 0, st, p);
        hipLaunchKernelGGL(mf_match_kernel<64>, g_match, dim3(256), 0, st, p);
        hipLaunchKernelGGL(mf_average_kernel<8>, g_avg, dim3(nt), lds, st, p);
    }
    return hipGetLastError();
}

}  // namespace pkv
