// Stages 2 and 3 of the PrefixKV hot path.
//
//  sort_prefix_kernel  one workgroup per (sequence, layer): the priority sequence of Sec. 3.2 (positions
//                      by importance, descending) by a bitonic sort of 64-bit keys -- in registers and
//                      wavefront shuffles wherever a stage stays inside a wavefront, through LDS otherwise --
//                      then the cumulative priority as an exact integer scan of fixed-point weights, and the
//                      layer's prefix lengths at the ratios t/256 (the first eight steps of the search).
//  search_kernel       one workgroup per sequence, 32 lanes per layer: Algorithm 1 (Sec. 3.3) runs to
//                      completion on the device -- eight steps on the summed tables, the rest on the
//                      cumulative sums -- followed by the proportional rescale to the budget.
//
// Everything that decides an index or a length is integer or a single fp64 product + compare, so the
// results do not depend on scan order or launch shape.
#include "pkv_common.hpp"

#include <mutex>

namespace pkv {

__device__ __forceinline__ uint64_t shfl_u64(uint64_t v, int src) {
    uint32_t lo = __shfl((uint32_t)v, src, kWave);
    uint32_t hi = __shfl((uint32_t)(v >> 32), src, kWave);
    return ((uint64_t)hi << 32) | lo;
}
// Sums never wrap: they stick at 2^62, far above the 2^53 limit that raises PKV_DEV_RANGE.
__device__ __forceinline__ uint64_t sat_add(uint64_t a, uint64_t b) {
    const uint64_t s = a + b, cap = 1ull << 62;
    return s > cap ? cap : s;
}
__device__ __forceinline__ uint64_t shfl_up_u64(uint64_t v, int d) {
    uint32_t lo = __shfl_up((uint32_t)v, d, kWave);
    uint32_t hi = __shfl_up((uint32_t)(v >> 32), d, kWave);
    return ((uint64_t)hi << 32) | lo;
}

// LDS written by lanes of one wavefront becomes visible to the other lanes of the same wavefront
__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Value of lane (l ^ J) for J = 1 .. 32 without a trip through the LDS crossbar: quad permutes (1, 2), row
// rotations (4, 8: a rotation by half a row of 16 is the exchange itself, by a quarter it is the exchange for
// one half of the lanes each way) and the 16- and 32-lane swaps of gfx950.
template <int J>
__device__ __forceinline__ uint32_t lane_xor(uint32_t x, int lane) {
    if constexpr (J == 1) return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0xB1, 0xF, 0xF, true);    // quad_perm [1,0,3,2]
    else if constexpr (J == 2) return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x4E, 0xF, 0xF, true);    // quad_perm [2,3,0,1]
    else if constexpr (J == 4) {
        const uint32_t dn = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x124, 0xF, 0xF, true);   // row_ror:4, from lane - 4
        const uint32_t up = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x12C, 0xF, 0xF, true);   // row_ror:12, from lane + 4
        return (lane & 4) ? dn : up;
    } else if constexpr (J == 8) return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x128, 0xF, 0xF, true);   // row_ror:8
    else if constexpr (J == 16) {
        const auto sw = __builtin_amdgcn_permlane16_swap(x, x, false, false);   // [r0 r0 r2 r2], [r1 r1 r3 r3]
        return (lane & 16) ? sw[0] : sw[1];
    } else {
        static_assert(J == 32, "lane distance");
        const auto sw = __builtin_amdgcn_permlane32_swap(x, x, false, false);   // [lo lo], [hi hi]
        return (lane & 32) ? sw[0] : sw[1];
    }
}
template <int J>
__device__ __forceinline__ uint64_t lane_xor_u64(uint64_t v, int lane) {
    const uint32_t lo = lane_xor<J>((uint32_t)v, lane), hi = lane_xor<J>((uint32_t)(v >> 32), lane);
    return ((uint64_t)hi << 32) | lo;
}

// The stages of bitonic merge step k whose partner distance is below 64*E, on keys held in registers: a
// wavefront owns an aligned block of 64*E keys, register e of lane l is position base + 64*e + l.  Distances
// of 64 and more pair two registers of one lane, smaller ones pair two lanes (one shuffle per key).
template <int E, int J>
__device__ __forceinline__ void lane_stage(uint64_t (&r)[E], int k, int base, int lane) {
    if (J >= k) return;
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const uint64_t a = r[e], b = lane_xor_u64<J>(a, lane);
        const bool up = ((base + 64 * e + lane) & k) == 0;
        const bool keep_min = ((lane & J) == 0) == up;
        r[e] = (a < b) == keep_min ? a : b;
    }
}
template <int E>
__device__ __forceinline__ void wave_stages(uint64_t (&r)[E], int k, int base, int lane) {
#pragma unroll
    for (int je = E / 2; je >= 1; je >>= 1) {           // partner distance 64*je, between registers
        if (64 * je >= k) continue;
#pragma unroll
        for (int e = 0; e < E; ++e) {
            if (e & je) continue;
            const bool up = ((base + 64 * e) & k) == 0; // lane < 64 <= k/2: the lane bits do not reach bit k
            const uint64_t a = r[e], b = r[e | je];
            const bool sw = (a > b) == up;
            r[e] = sw ? b : a;
            r[e | je] = sw ? a : b;
        }
    }
    lane_stage<E, 32>(r, k, base, lane);                // between lanes
    lane_stage<E, 16>(r, k, base, lane);
    lane_stage<E, 8>(r, k, base, lane);
    lane_stage<E, 4>(r, k, base, lane);
    lane_stage<E, 2>(r, k, base, lane);
    lane_stage<E, 1>(r, k, base, lane);
}

// Ratios served from a table: p = (t + 1) / 2^kTabBits, t = 0 .. kTabN - 1 (rows of kTabN + 1 ints)
constexpr int kTabBits = 8;
constexpr int kTabN = (1 << kTabBits) - 1;

// Sort key: high word = ~bits(importance) (non-negative floats order like their bit patterns, so the
// complement orders them descending), low word = position (ascending among equal values).
// Padding keys are all ones: they sort last and decode to weight 0.
// P = E * ns keys, ns = the sorting threads (whole wavefronts, the first of the workgroup); a bitonic network,
// ascending.  Merge steps up to 64*E keys and the tail of every longer one run in registers inside a
// wavefront, without a barrier; only the stages that pair keys of different wavefronts go through LDS.
template <int E>
__global__ void sort_prefix_kernel(int N, int P, const float* __restrict__ importance,
                                   int32_t* __restrict__ order, uint64_t* __restrict__ cum,
                                   float* __restrict__ prefix, int32_t* __restrict__ seg_status,
                                   int32_t* __restrict__ ktab) {
    extern __shared__ uint64_t skey[];          // P keys, then reused for the scan
    __shared__ uint64_t wave_tot[16];
    __shared__ int s_flags;
    const int tid = threadIdx.x, nt = P / E;    // nt sorting threads; a larger workgroup idles the rest
    const int lane = tid & (kWave - 1), wv = tid / kWave;
    const bool sorter = tid < nt;
    const size_t seg = blockIdx.x;
    const float* imp = importance + seg * (size_t)N;
    if (tid == 0) s_flags = 0;

    int flags = 0;
    const int wbase = wv * (kWave * E);
    uint64_t r[E];
    if (sorter) {
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const int i = wbase + kWave * e + lane;
            uint64_t key = ~0ull;
            if (i < N) {
                uint32_t bits = __float_as_uint(imp[i]);
                if ((bits & 0x7f800000u) == 0x7f800000u) flags |= PKV_DEV_NONFINITE;
                else if (bits == 0x80000000u) bits = 0;  // -0.0 counts as +0.0
                else if (bits & 0x80000000u) flags |= PKV_DEV_NEGATIVE;
                key = ((uint64_t)(~bits) << 32) | (uint32_t)i;
            }
            r[e] = key;
        }
        const int kw = P < kWave * E ? P : kWave * E;
        for (int k = 2; k <= kw; k <<= 1) wave_stages<E>(r, k, wbase, lane);
    }
    __syncthreads();                                      // s_flags = 0 is visible
    if (flags) atomicOr(&s_flags, flags);
    for (int k = 2 * kWave * E; k <= P; k <<= 1) {
        if (sorter) {
#pragma unroll
            for (int e = 0; e < E; ++e) skey[wbase + kWave * e + lane] = r[e];
        }
        __syncthreads();
        for (int j = k >> 1; j >= kWave * E; j >>= 1) {
            for (int t = tid; t < (P >> 1); t += blockDim.x) {
                const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
                const int x = i | j;
                const uint64_t a = skey[i], b = skey[x];
                const bool up = (i & k) == 0;
                if ((a > b) == up) { skey[i] = b; skey[x] = a; }
            }
            __syncthreads();
        }
        if (sorter) {
#pragma unroll
            for (int e = 0; e < E; ++e) r[e] = skey[wbase + kWave * e + lane];
            wave_stages<E>(r, k, wbase, lane);
        }
        // the next write of skey (next k, or the sorted keys below) is to this wavefront's own block, which
        // only this wavefront has read since the last barrier
    }
    if (sorter) {
#pragma unroll
        for (int e = 0; e < E; ++e) skey[wbase + kWave * e + lane] = r[e];
    }
    __syncthreads();

    // fixed-point weights and their inclusive scan; each thread owns E consecutive sorted entries
    const int base = tid * E;                 // threads beyond the sorting ones own nothing
    uint64_t local = 0;
    const double two36 = 68719476736.0;
    flags = 0;                                // what the key pass found is in s_flags already
    for (int e = 0; e < (sorter ? E : 0); ++e) {
        const uint64_t key = skey[base + e];
        const float v = __uint_as_float(~(uint32_t)(key >> 32));
        const double wd = floor((double)v * two36);
        uint64_t w = 0;
        if (base + e < N) {
            if (wd >= 9007199254740992.0) flags |= PKV_DEV_RANGE; else w = (uint64_t)wd;
            order[seg * (size_t)N + base + e] = (int32_t)(uint32_t)key;
        }
        local = sat_add(local, w);
        skey[base + e] = local;  // thread-local inclusive sums, rebased below
    }
    // scan of the thread totals: within the wave by shuffles, across waves through LDS
    uint64_t incl = local;
    for (int d = 1; d < kWave; d <<= 1) {
        const uint64_t up = shfl_up_u64(incl, d);
        if (lane >= d) incl = sat_add(incl, up);
    }
    if (lane == kWave - 1) wave_tot[wv] = incl;
    __syncthreads();
    uint64_t wave_base = 0, total = 0;
    const int nw = nt / kWave;
    for (int w = 0; w < nw; ++w) {
        const uint64_t t = wave_tot[w];
        if (w < wv) wave_base = sat_add(wave_base, t);
        total = sat_add(total, t);
    }
    const uint64_t excl = sat_add(wave_base, incl - local);
    if (total > (1ull << 53)) flags |= PKV_DEV_RANGE;
    if (flags) atomicOr(&s_flags, flags);
    const double dtotal = (double)total;
    for (int e = 0; e < E; ++e) {
        const int j = base + e;
        if (j < N) {
            const uint64_t c = sat_add(excl, skey[j]);
            cum[seg * (size_t)N + j] = c;
            skey[j] = c;
            if (prefix && total) prefix[seg * (size_t)N + j] = (float)((double)c / dtotal);
        }
    }
    __syncthreads();
    // The first kTabBits steps of Algorithm 1 (Sec. 3.3) can only ask for the ratios t / 2^kTabBits: the prefix
    // length of this layer at each of them, from the row while it is still in LDS.  The search adds the
    // layers' tables up and walks those steps without touching the rows.
    if (ktab) {
        for (int t = tid; t < kTabN; t += blockDim.x) {
            const double thr = __dmul_rn((double)(t + 1) * (1.0 / (double)(kTabN + 1)), dtotal);
            int lo = 1, hi = N;                           // smallest k in [1, N] with C_k >= thr (C_N >= thr)
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if ((double)skey[mid - 1] >= thr) hi = mid; else lo = mid + 1;
            }
            ktab[seg * (size_t)(kTabN + 1) + t] = lo;
        }
    }
    if (tid == 0) {
        // invalid values win over a range overflow, which wins over an all-zero layer
        int f = s_flags;
        if (f & (PKV_DEV_NONFINITE | PKV_DEV_NEGATIVE)) f &= (PKV_DEV_NONFINITE | PKV_DEV_NEGATIVE);
        else if (f & PKV_DEV_RANGE) f = PKV_DEV_RANGE;
        else if (total == 0) f = PKV_DEV_ZERO_LAYER;
        seg_status[seg] = f;
    }
}

// Proportional rescale of per-layer weights to an exact token budget, by one wavefront (lane l = layer l):
// out[l] = weight_l * budget / K rounded down and clamped to [1, N]; the missing tokens go one per layer in
// order of largest remainder (ties: lower layer), cyclically; a surplus is taken back by smallest remainder.
// Whole rounds of the cyclic walk are applied at once while no layer can hit its limit, the last partial
// round visits in rank order: equal to the one-token-at-a-time walk.  Requires L < budget < L*N, K > 0.
// `out` may be global or shared memory; s_sorted / s_len are kMaxL ints of shared scratch.
__device__ __forceinline__ void rescale_wave(int L, int N, uint64_t weight, uint64_t K, int64_t budget,
                                             int32_t* out, int* s_sorted, int* s_len) {
    const int lane = threadIdx.x;
    const bool act = lane < L;
    const uint64_t num = act ? weight * (uint64_t)budget : 0;
    int64_t bs = (int64_t)(num / K);
    bs = bs < 1 ? 1 : (bs > N ? N : bs);
    const uint64_t rem = num % K;
    int sumb = act ? (int)bs : 0;
    for (int d = 32; d > 0; d >>= 1) sumb += __shfl_xor(sumb, d, kWave);
    int64_t dlt = budget - sumb;
    const bool grow = dlt > 0;
    int rank = 0;
    for (int j = 0; j < L; ++j) {
        const uint64_t rj = shfl_u64(rem, j);
        const bool before = grow ? (rj > rem || (rj == rem && j < lane))
                                 : (rj < rem || (rj == rem && j < lane));
        rank += before ? 1 : 0;
    }
    wave_sync();
    if (act) { s_sorted[rank] = lane; s_len[lane] = (int)bs; }
    wave_sync();
    if (lane == 0 && dlt != 0) {
        int64_t left = grow ? dlt : -dlt;
        while (left > 0) {
            int elig = 0;
            int64_t room = N;
            for (int i = 0; i < L; ++i) {
                const int v = s_len[i];
                const int r = grow ? N - v : v - 1;
                if (r > 0) { ++elig; room = r < room ? r : room; }
            }
            if (elig == 0) break;  // cannot happen for L < budget < L*N
            if (left >= elig) {
                int64_t rounds = left / elig;
                if (rounds > room) rounds = room;
                for (int i = 0; i < L; ++i) {
                    const int v = s_len[i];
                    if ((grow ? N - v : v - 1) > 0) s_len[i] = v + (grow ? (int)rounds : -(int)rounds);
                }
                left -= rounds * elig;
            } else {
                for (int i = 0; i < L && left > 0; ++i) {
                    const int l = s_sorted[i];
                    const int v = s_len[l];
                    if ((grow ? N - v : v - 1) > 0) { s_len[l] = v + (grow ? 1 : -1); --left; }
                }
            }
        }
    }
    wave_sync();
    const int res = act ? s_len[lane] : 0;
    wave_sync();
    if (act) out[lane] = res;
}

// Algorithm 1 (Sec. 3.3) for one sequence per workgroup.  A group of 32 lanes owns a layer (two layers when
// L > 32); p1, p2, p live in every thread with identical arithmetic, so control flow stays uniform and no
// iteration leaves the device.  The prefix length of a layer at ratio p is the smallest k with C_k >= p*T
// inside the bracket [k_lo, k_hi] left by the earlier iterations (the length is monotone in p).  Because the
// cumulative sums ascend, any search order gives that same k; a group finds it 32 entries at a time instead of
// one: 32 probes spread over the whole row are read once and kept in registers (they narrow every later
// threshold to 1/33 of the row without a load), wider remainders are probed again, and the last 32 candidates
// are held as a window that is reused as long as the bracket stays inside it.  Per iteration this costs one
// dependent load or none, instead of log2(bracket).
constexpr int kSearchGroup = 32;
constexpr int kSearchThreads = 1024;

struct LayerSearch {
    const uint64_t* c;       // c[k-1] = C_k
    int k_lo, k_hi, k;
    int cstep_w;             // N - 1 when the coarse probes exist, else 0
    double cval;             // coarse probe of this lane: C at 1 + ((j+1) * (N-1)) / 33
    int wbase;               // window: lane j holds C_{wbase + j}; wbase = 0: empty
    double wval;             // (the sums stay below 2^53, so they are exact as doubles)
};

__device__ __forceinline__ uint32_t ballot32(bool pred, int lane) {
    const unsigned long long m = __builtin_amdgcn_ballot_w64(pred);
    return (uint32_t)(m >> (lane & 32));
}

// smallest k in [k_lo, k_hi) with (double)C_k >= thr, k_hi if there is none; uniform within the 32-lane group
__device__ __forceinline__ int search_layer(LayerSearch& s, double thr, int N, int lane) {
    const int j = lane & 31;
    int a = s.k_lo, e = s.k_hi;
    // once the bracket lies inside the window, an iteration is one compare and one ballot
    const bool inside = s.wbase != 0 && a >= s.wbase && e <= s.wbase + kSearchGroup;
    if (!inside) {
        if (s.cstep_w) {
            const int kc = 1 + ((j + 1) * s.cstep_w) / 33;
            const bool in = kc >= a && kc < e, ge = s.cval >= thr;
            const uint32_t m_ge = ballot32(in && ge, lane), m_lt = ballot32(in && !ge, lane);
            if (m_ge) e = 1 + ((__builtin_ctz(m_ge) + 1) * s.cstep_w) / 33;
            if (m_lt) a = 2 + ((32 - __builtin_clz(m_lt)) * s.cstep_w) / 33;
        }
        while (e - a > kSearchGroup) {
            const int width = e - a;
            const int kj = a + ((j + 1) * width) / 33;              // a < kj < e, ascending in j
            const bool ge = (double)s.c[kj - 1] >= thr;
            const uint32_t m_ge = ballot32(ge, lane);
            if (m_ge == 0) {
                a = a + (32 * width) / 33 + 1;
            } else {
                const int js = __builtin_ctz(m_ge);
                e = a + ((js + 1) * width) / 33;
                if (js > 0) a = a + (js * width) / 33 + 1;
            }
        }
        if (a < e && (s.wbase == 0 || a < s.wbase || e > s.wbase + kSearchGroup)) {
            // anchor the window at the bracket when it already fits: every later search stays inside it
            s.wbase = s.k_hi - s.k_lo <= kSearchGroup ? s.k_lo : a;
            s.wval = s.wbase + j <= N ? (double)s.c[s.wbase + j - 1] : INFINITY;
        }
    }
    if (a < e) {
        const int kk = s.wbase + j;
        const uint32_t m = ballot32(kk >= a && kk < e && s.wval >= thr, lane);
        if (m) e = s.wbase + __builtin_ctz(m);
    }
    return e;
}

__global__ void __launch_bounds__(kSearchThreads)
search_kernel(int L, int N, const uint64_t* __restrict__ cum, const int32_t* __restrict__ seg_status,
              const int32_t* __restrict__ ktab, int64_t budget, int64_t tol, int max_iters, int fixup, int32_t* __restrict__ lengths,
              double* __restrict__ p_out, int32_t* __restrict__ iters_out,
              int64_t* __restrict__ raw_total_out, int32_t* __restrict__ status) {
    __shared__ int s_sorted[kMaxL];
    __shared__ int s_len[kMaxL];
    __shared__ int s_k[2][kMaxL];
    __shared__ int s_sum[3];     // total length of iteration it in s_sum[it % 3]
    __shared__ int s_st;
    __shared__ int s_ktot[kTabN + 1];
    __shared__ unsigned long long s_below[(kTabN + 1) / 64], s_hit[(kTabN + 1) / 64];
    extern __shared__ int s_tab[];                        // with a table: the sequence's L rows of kTabN + 1 ints
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & (kWave - 1);
    const int grp = tid / kSearchGroup, ngrp = blockDim.x / kSearchGroup;
    const bool tab = ktab != nullptr;
    // The layers of this group: grp and grp + ngrp (ngrp >= min(L, 32), L <= 64).  Their totals and coarse
    // probes are requested here, together with the table and ahead of the status, so that the kernel starts
    // with one round trip to memory instead of three (the rows of a refused layer hold unspecified but
    // readable values).
    LayerSearch ls[2];
    double T[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int l = grp + i * ngrp;
        const bool act = l < L;
        ls[i].c = cum + ((size_t)b * L + (act ? l : 0)) * (size_t)N;
        ls[i].k_lo = 1; ls[i].k_hi = N; ls[i].k = 1; ls[i].wbase = 0; ls[i].wval = 0.0;
        ls[i].cstep_w = N - 1 > kSearchGroup ? N - 1 : 0;
        ls[i].cval = 0.0;
        T[i] = 0.0;
        if (act) {
            T[i] = (double)ls[i].c[N - 1];
            if (ls[i].cstep_w) ls[i].cval = (double)ls[i].c[((lane & 31) + 1) * ls[i].cstep_w / 33];   // C at 1 + that
        }
    }
    // the table of the sequence into LDS (read before the status is known: the row of a refused layer holds
    // some in-range integers, and is not used)
    if (tab) {
        const int4* src = (const int4*)(ktab + (size_t)b * L * (kTabN + 1));
        for (int i = tid; i < L * (kTabN + 1) / 4; i += blockDim.x) ((int4*)s_tab)[i] = src[i];
    }
    const int st_mine = tid < L ? seg_status[(size_t)b * L + tid] : 0;
    if (tid == 0) { s_st = 0; s_sum[0] = 0; s_sum[1] = 0; s_sum[2] = 0; }
    __syncthreads();
    if (st_mine) atomicOr(&s_st, st_mine);
    if (tab) {
        // Total length of the sequence at every tabulated ratio, and how it compares with the budget: one bit
        // per ratio for "below the budget by more than the tolerance" and one for "within the tolerance".
        // The tabulated steps of the search then only test bits.
        for (int t0 = 0; t0 <= kTabN; t0 += blockDim.x) {         // whole wavefronts: a wavefront = one mask word
            const int t = t0 + tid;
            int sum = 0;
            if (t < kTabN)
                for (int l = 0; l < L; ++l) sum += s_tab[l * (kTabN + 1) + t];
            const int64_t d = (int64_t)sum - budget;
            const unsigned long long mb = __builtin_amdgcn_ballot_w64(t < kTabN && d < -tol);
            const unsigned long long mh = __builtin_amdgcn_ballot_w64(t < kTabN && (d < 0 ? -d : d) <= tol);
            if (t <= kTabN) {
                s_ktot[t] = sum;
                if (lane == 0) { s_below[t >> 6] = mb; s_hit[t >> 6] = mh; }
            }
        }
    }
    __syncthreads();
    const int st = s_st;
    if (st) {
        if (tid < L) lengths[(size_t)b * L + tid] = 0;
        if (tid == 0) { p_out[b] = 0.0; iters_out[b] = 0; raw_total_out[b] = 0; status[b] = st; }
        return;
    }
    if (budget <= L || budget >= (int64_t)L * N) {
        const bool all = budget > L;
        if (tid < L) lengths[(size_t)b * L + tid] = all ? N : 1;
        if (tid == 0) {
            p_out[b] = all ? 1.0 : 0.0; iters_out[b] = 0;
            raw_total_out[b] = all ? (int64_t)L * N : L; status[b] = 0;
        }
        return;
    }

    double p1 = 0.0, p2 = 1.0, p = 0.5;
    int iters = 0, K = 0, it0 = 1;
    if (tab) {
        // the tabulated steps: every thread walks them alike (s_ktot is complete since the status barrier)
        int t_lo = -1, t_hi = kTabN, t_last = -1;         // table columns of p1, p2 (none for 0 and 1) and p
        bool stop = false;
        unsigned long long below[(kTabN + 1) / 64], hit[(kTabN + 1) / 64];
#pragma unroll
        for (int w = 0; w < (kTabN + 1) / 64; ++w) { below[w] = s_below[w]; hit[w] = s_hit[w]; }
        for (; it0 <= max_iters && it0 <= kTabBits; ++it0) {
            // p = (p1 + p2) / 2 is a multiple of 2^-it0, never equal to p1 or p2; its column is the middle of
            // the columns of p1 and p2
            t_last = (t_lo + t_hi) >> 1;
            iters = it0;
            unsigned long long wb = below[0], wh = hit[0];
#pragma unroll
            for (int w = 1; w < (kTabN + 1) / 64; ++w)
                if ((t_last >> 6) == w) { wb = below[w]; wh = hit[w]; }
            if ((wh >> (t_last & 63)) & 1) { stop = true; break; }
            if ((wb >> (t_last & 63)) & 1) t_lo = t_last; else t_hi = t_last;
        }
        // the ratios as Algorithm 1 would hold them: exact dyadic numbers
        p1 = (double)(t_lo + 1) * (1.0 / (double)(kTabN + 1));
        p2 = (double)(t_hi + 1) * (1.0 / (double)(kTabN + 1));
        p = (double)(t_last + 1) * (1.0 / (double)(kTabN + 1));
        K = s_ktot[t_last];
        if (stop || it0 > max_iters) {                    // ended inside the table
            if (tid == 0) { p_out[b] = p; iters_out[b] = iters; raw_total_out[b] = K; status[b] = 0; }
            const int k_mine = tid < L ? s_tab[tid * (kTabN + 1) + t_last] : 0;
            if (!fixup || K == budget) {
                if (tid < L) lengths[(size_t)b * L + tid] = k_mine;
                return;
            }
            if (tid < kWave)
                rescale_wave(L, N, tid < L ? (uint64_t)k_mine : 0, (uint64_t)K, budget, lengths + (size_t)b * L, s_sorted, s_len);
            return;
        }
        // the brackets the earlier steps would have left: the lengths at p1 and p2
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int l = grp + i * ngrp;
            if (l < L) {
                if (t_lo >= 0) ls[i].k_lo = s_tab[l * (kTabN + 1) + t_lo];
                if (t_hi < kTabN) ls[i].k_hi = s_tab[l * (kTabN + 1) + t_hi];
            }
        }
    }
    for (int it = it0; it <= max_iters; ++it) {
        const double mid = 0.5 * (p1 + p2);
        if (mid == p1 || mid == p2) break;
        p = mid;
        int* sk = s_k[it & 1];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int l = grp + i * ngrp;
            if (l < L) {                                  // uniform within the group
                const double thr = __dmul_rn(p, T[i]);    // one rounded product, never contracted
                ls[i].k = search_layer(ls[i], thr, N, lane);
                if ((lane & 31) == 0) { sk[l] = ls[i].k; atomicAdd(&s_sum[it % 3], ls[i].k); }
            }
        }
        __syncthreads();
        K = s_sum[it % 3];
        if (tid == 0) s_sum[(it + 2) % 3] = 0;            // next used two iterations from now, after another barrier
        iters = it;
        const int64_t delta = (int64_t)K - budget;
        if ((delta < 0 ? -delta : delta) <= tol) break;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            if (delta < 0) ls[i].k_lo = ls[i].k; else ls[i].k_hi = ls[i].k;
        }
        if (delta < 0) p1 = p; else p2 = p;
    }
    if (tid == 0) { p_out[b] = p; iters_out[b] = iters; raw_total_out[b] = K; status[b] = 0; }
    if (iters == 0) {                                     // max_iters < 1 cannot happen (checked by the caller)
        if (tid < L) lengths[(size_t)b * L + tid] = 1;
        return;
    }
    // s_k[iters & 1] holds the lengths of the last iteration; every thread has passed its barrier
    const int k_mine = tid < L ? s_k[iters & 1][tid] : 0;
    if (!fixup || K == budget) {
        if (tid < L) lengths[(size_t)b * L + tid] = k_mine;
        return;
    }
    if (tid < kWave)                                      // one wavefront, lane l = layer l
        rescale_wave(L, N, tid < L ? (uint64_t)k_mine : 0, (uint64_t)K, budget, lengths + (size_t)b * L, s_sorted, s_len);
}

// Offline configuration (Sec. 3.3, last paragraph): the lengths of S calibration sequences are summed per
// layer (averaging the per-sample ratios R_l) and rescaled to the budget of the deployed prompt length N.
// One wavefront; the same row is written `copies` times so that it can be used as a [B,L] lengths array.
__global__ void __launch_bounds__(kWave)
offline_config_kernel(int S, int L, int N, const int32_t* __restrict__ sample_lengths, int64_t budget,
                      int copies, int32_t* __restrict__ lengths) {
    __shared__ int s_sorted[kMaxL];
    __shared__ int s_len[kMaxL];
    const int lane = threadIdx.x;
    const bool act = lane < L;
    long long w = 0;
    if (act)
        for (int s = 0; s < S; ++s) w += sample_lengths[(size_t)s * L + lane];
    long long K = w;
    for (int d = 32; d > 0; d >>= 1) {
        const uint32_t lo = __shfl_xor((uint32_t)K, d, kWave);
        const uint32_t hi = __shfl_xor((uint32_t)((unsigned long long)K >> 32), d, kWave);
        K += (long long)(((unsigned long long)hi << 32) | lo);
    }
    const bool trivial = K == 0 || budget <= L || budget >= (int64_t)L * N;
    if (trivial) {
        if (act) s_len[lane] = K == 0 ? 0 : (budget <= L ? 1 : N);
    } else {
        rescale_wave(L, N, (uint64_t)w, (uint64_t)K, budget, s_len, s_sorted, s_len);
    }
    __syncthreads();
    if (act)
        for (int c = 0; c < copies; ++c) lengths[(size_t)c * L + lane] = s_len[lane];
}

// Per-sequence status word = OR of its layers' status words (used when stage 2 runs without the search).
__global__ void __launch_bounds__(kWave)
status_reduce_kernel(int L, const int32_t* __restrict__ seg_status, int32_t* __restrict__ status) {
    const int b = blockIdx.x, lane = threadIdx.x;
    int st = lane < L ? seg_status[(size_t)b * L + lane] : 0;
    for (int d = 32; d > 0; d >>= 1) st |= __shfl_xor(st, d, kWave);
    if (lane == 0) status[b] = st;
}

// Gini coefficient of every layer's priority sequence (Sec. 4.3): G = (2 * sum_k C_k / C_N - N - 1) / N on the
// exact cumulative sums.  sum_k C_k can reach 2^66, so it is kept as a (high, low) pair of 64-bit words; the
// per-thread pairs are added up in thread order by one thread.
__global__ void __launch_bounds__(256)
gini_kernel(int N, const uint64_t* __restrict__ cum, double* __restrict__ gini) {
    __shared__ uint64_t s_lo[256], s_hi[256];
    const uint64_t* c = cum + (size_t)blockIdx.x * N;
    uint64_t lo = 0, hi = 0;
    for (int i = threadIdx.x; i < N; i += 256) {
        const uint64_t a = c[i], t = lo + a;
        hi += t < lo ? 1 : 0;
        lo = t;
    }
    s_lo[threadIdx.x] = lo; s_hi[threadIdx.x] = hi;
    __syncthreads();
    if (threadIdx.x == 0) {
        lo = 0; hi = 0;
        for (int i = 0; i < 256; ++i) {
            const uint64_t t = lo + s_lo[i];
            hi += s_hi[i] + (t < lo ? 1 : 0);
            lo = t;
        }
        const double S = (double)hi * 18446744073709551616.0 + (double)lo;
        const double T = (double)c[N - 1];
        gini[blockIdx.x] = T > 0.0 ? (2.0 * (S / T) - (double)N - 1.0) / (double)N : 0.0;
    }
}

static int pow2_at_least(int n) { int p = 64; while (p < n) p <<= 1; return p; }

// one workgroup per segment; keys per thread: 1 for up to 64 keys, 2 up to 2048, then 4 and 8 (1024 threads).
// (Fewer, fatter wavefronts -- four with P / 256 keys per lane -- were slower: 9.2 us against 7.7 us for the
// sort at N = 680; a stage is bound by the latency of its shuffle, which more wavefronts hide.)
template <int E>
static hipError_t launch_sort_prefix_e(int nseg, int N, int P, const float* importance, int32_t* order,
                                       uint64_t* cum, float* prefix, int32_t* seg_status, int32_t* ktab,
                                       hipStream_t st) {
    const size_t lds = (size_t)P * sizeof(uint64_t);
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void*)sort_prefix_kernel<E>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(sort_prefix_kernel<E>, dim3(nseg), dim3(P / E), lds, st, N, P, importance, order, cum,
                       prefix, seg_status, ktab);
    return hipGetLastError();
}
static hipError_t launch_sort_prefix(int nseg, int N, const float* importance, int32_t* order, uint64_t* cum,
                                     float* prefix, int32_t* seg_status, int32_t* ktab, hipStream_t st) {
    const int P = pow2_at_least(N);
    if (P <= 64) return launch_sort_prefix_e<1>(nseg, N, P, importance, order, cum, prefix, seg_status, ktab, st);
    if (P <= 2048) return launch_sort_prefix_e<2>(nseg, N, P, importance, order, cum, prefix, seg_status, ktab, st);
    if (P <= 4096) return launch_sort_prefix_e<4>(nseg, N, P, importance, order, cum, prefix, seg_status, ktab, st);
    if (P <= 8192) return launch_sort_prefix_e<8>(nseg, N, P, importance, order, cum, prefix, seg_status, ktab, st);
    return hipErrorInvalidValue;
}

// a status word per segment, then (256-byte aligned) a table row per segment
static size_t select_tab_offset(int B, int L) { return ((size_t)B * L * sizeof(int32_t) + 255) / 256 * 256; }
size_t select_ws_bytes(int B, int L, int N) {
    (void)N;
    return select_tab_offset(B, L) + (size_t)B * L * (kTabN + 1) * sizeof(int32_t);
}

hipError_t launch_select(int B, int L, int N, const float* importance, const pkv_select_params& pr,
                         int32_t* order, uint64_t* cum, float* prefix, int32_t* lengths, double* p_out,
                         int32_t* iters, int64_t* raw_total, int32_t* status, void* ws, bool with_table,
                         hipStream_t st) {
    int32_t* seg_status = (int32_t*)ws;
    int32_t* ktab = with_table ? (int32_t*)((unsigned char*)ws + select_tab_offset(B, L)) : nullptr;
    hipError_t e = launch_sort_prefix(B * L, N, importance, order, cum, prefix, seg_status, ktab, st);
    if (e != hipSuccess) return e;
    // one 32-lane group per layer (two layers per group beyond 32), whole wavefronts
    int search_threads = (L * kSearchGroup + kWave - 1) / kWave * kWave;
    if (search_threads > kSearchThreads) search_threads = kSearchThreads;
    const size_t tab_lds = ktab ? (size_t)L * (kTabN + 1) * sizeof(int32_t) : 0;
    if (tab_lds > 32 * 1024) {
        e = hipFuncSetAttribute((const void*)search_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)tab_lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(search_kernel, dim3(B), dim3(search_threads), tab_lds, st, L, N, cum, seg_status, ktab,
                       (int64_t)pr.budget_tokens, (int64_t)pr.tol_tokens, (int)pr.max_iters, (int)pr.fixup,
                       lengths, p_out, iters, raw_total, status);
    return hipGetLastError();
}

// ---- prefixkv_select for callers that cannot allocate: the per-layer status words live in a
// file-scope device array instead of a caller workspace.  Every GPU holds its own copy of the array at
// its own address; that address is looked up once per device (the array's name is only a host-side
// handle and must never be passed to a kernel).  Nothing in the array has to start at zero:
// sort_prefix_kernel writes the word of every segment of the call before search_kernel reads it.
constexpr int kStaticSegments = 65536;                 // B * L of one call at most (256 KB per GPU)
constexpr int kStaticMaxDevices = 64;
static __device__ __align__(256) int32_t scratch[kStaticSegments];

namespace {
std::mutex g_scratch_mutex;
int32_t* g_scratch_ptr[kStaticMaxDevices] = {};         // device address of `scratch`, per device ordinal
}  // namespace

int select_static_max_segments() { return kStaticSegments; }

hipError_t launch_select_static(int B, int L, int N, const float* importance, const pkv_select_params& pr,
                                int32_t* order, uint64_t* cum, float* prefix, int32_t* lengths, double* p_out,
                                int32_t* iters, int64_t* raw_total, int32_t* status, hipStream_t st) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kStaticMaxDevices) return hipErrorInvalidDevice;
    int32_t* ptr = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (g_scratch_ptr[dev] == nullptr) {            // first call on this device, which is current
            void* p = nullptr;
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e != hipSuccess) return e;
            if (p == nullptr) return hipErrorInvalidSymbol;
            g_scratch_ptr[dev] = (int32_t*)p;
        }
        ptr = g_scratch_ptr[dev];
    }
    // no table here: a status word is all a segment needs, the search walks every step on the rows
    return launch_select(B, L, N, importance, pr, order, cum, prefix, lengths, p_out, iters, raw_total, status,
                         ptr, false, st);
}

hipError_t launch_rank(int B, int L, int N, const float* importance, int32_t* order, uint64_t* cum,
                       float* prefix, int32_t* status, void* ws, hipStream_t st) {
    int32_t* seg_status = (int32_t*)ws;
    hipError_t e = launch_sort_prefix(B * L, N, importance, order, cum, prefix, seg_status, nullptr, st);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(status_reduce_kernel, dim3(B), dim3(kWave), 0, st, L, seg_status, status);
    return hipGetLastError();
}

hipError_t launch_offline_config(int S, int L, int N, const int32_t* sample_lengths, int64_t budget,
                                 int copies, int32_t* lengths, hipStream_t st) {
    hipLaunchKernelGGL(offline_config_kernel, dim3(1), dim3(kWave), 0, st, S, L, N, sample_lengths, budget,
                       copies, lengths);
    return hipGetLastError();
}

hipError_t launch_gini(int B, int L, int N, const uint64_t* cum, double* gini, hipStream_t st) {
    hipLaunchKernelGGL(gini_kernel, dim3(B * L), dim3(256), 0, st, N, cum, gini);
    return hipGetLastError();
}

}  // namespace pkv
