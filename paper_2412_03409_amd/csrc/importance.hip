// Stage 1: KV importance (Sec. 3.2) -- column sums of the causal softmax, averaged over heads.
//
// bf16 inputs run on the matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulate) in ONE kernel that reads
// the queries and the keys of a head from HBM once (importance_fused_kernel, below): the queries stay in
// registers, the keys stream through LDS twice -- first for the row log-sum-exp, then for the column sums --
// and swapping the MFMA operands between the two sweeps gives the layout each of them wants: a lane holds one
// query and 16 keys in the first (the running max / sum of a row is a scalar per lane), one key and 16 queries
// in the second (the column sum of a key is a sum inside the lane).
//
// The head mean is a second, tiny kernel that adds the per-workgroup partial sums in (head, workgroup)
// order, so the result is bitwise reproducible.  fp32 inputs (small validation shapes) use plain kernels.
#include "pkv_common.hpp"

namespace pkv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr int kStage = 128;   // streamed rows per LDS stage

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

// Accumulator register r of lane `lane` holds row 8*(r/4) + 4*(lane/32) + r%4, column lane%32 of
// the 32x32 product.
__device__ __forceinline__ int acc_row(int r, int lane) { return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }

// ---- staging of a streamed kStage-row tile: global memory -> LDS without passing through registers ------
// gfx950's 16-byte global-to-LDS load writes lane i's 16 bytes to LDS[base + 16*i] (base is uniform per
// wavefront), i.e. one instruction fills 1 KB of consecutive LDS; each lane may fetch any global address.
// The tile is stored unpadded, rows of D bf16, with the 16-byte chunks of a row XOR-swizzled by the row
// index so that the MFMA fragment reads (32 rows x one chunk) hit all banks evenly:
//   chunk c of row r lives at chunk position c ^ ((r / RPB) & (CPR-1)),  RPB = rows per 256 bytes.
typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(1))) const void glb_void_t;

template <int D, int WV = 4> struct Stage {
    static constexpr int CPR = D / 8;                 // 16-byte chunks per row
    static constexpr int ROWB = D * 2;                // bytes per row
    static constexpr int RPB = 256 / ROWB;            // rows per 256 bytes (one pass over the 64 banks)
    static constexpr int BYTES = kStage * ROWB;
    static constexpr int PIECES = BYTES / 1024;       // 1 KB pieces of the tile, dealt to the wavefronts in turn
    static constexpr int INSTS = (PIECES + WV - 1) / WV;
    // Issue the asynchronous copy of rows [row0, row0 + kStage) (clamped to N-1) into `lds`.
    static __device__ __forceinline__ void issue(const bf16_t* base, int64_t ld, int row0, int N,
                                                 unsigned char* lds, int wv, int lane) {
        // the per-lane address pieces are recomputed at every call (a few integer operations per stage): kept
        // across a long loop they would occupy two dozen registers
        asm volatile("" : "+v"(lane));
#pragma unroll
        for (int i = 0; i < INSTS; ++i) {
            const int inst = i * WV + wv;             // which 1 KB piece of the tile
            if (PIECES % WV != 0 && inst >= PIECES) break;
            const int L = inst * 64 + lane;           // linear chunk index in LDS
            const int row = L / CPR, pos = L % CPR;
            const int c = pos ^ ((row / RPB) & (CPR - 1));
            int grow = row0 + row;
            grow = grow < N ? grow : N - 1;
            // 32-bit element offset from the uniform base of this head (N * ld < 2^31, checked by the launcher)
            const bf16_t* g = base + ((uint32_t)grow * (uint32_t)ld + (uint32_t)(c * 8));
            __builtin_amdgcn_global_load_lds((glb_void_t*)g, (lds_void_t*)(lds + inst * 1024), 16, 0, 0);
        }
    }
    // MFMA operand fragment for k-step kk of the 32 rows starting at row0 (a multiple of 32)
    static __device__ __forceinline__ bf16x8 frag(const unsigned char* lds, int row0, int kk, int lane) {
        const int r = lane & 31;
        const int pos = (2 * kk + (lane >> 5)) ^ ((r / RPB) & (CPR - 1));
        return as_bf16x8(*(const uint4*)(lds + (row0 + r) * ROWB + pos * 16));
    }
};
// wait until this wavefront's global-to-LDS copies have landed (vmcnt = 0; other counters untouched)
__device__ __forceinline__ void wait_async_copies() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// The wavefront's stationary operand: two tiles of 32 rows (starting at row0 and row1), straight from global memory into the MFMA
// register layout.  flip = the rows are negated (exact in bf16) so that the logit scale is positive.
template <int D>
__device__ __forceinline__ void load_stationary(bf16x8 (&f)[2][D / 16], const bf16_t* base, int64_t ld, int row0,
                                                int row1, int N, int lane, bool flip) {
    const uint32_t sgn = flip ? 0x80008000u : 0u;
#pragma unroll
    for (int a = 0; a < 2; ++a) {
        int row = (a == 0 ? row0 : row1) + (lane & 31);
        row = row < N ? row : N - 1;
#pragma unroll
        for (int kk = 0; kk < D / 16; ++kk) {
            uint4 v = *(const uint4*)(base + (int64_t)row * ld + 16 * kk + 8 * (lane >> 5));
            v.x ^= sgn; v.y ^= sgn; v.z ^= sgn; v.w ^= sgn;
            f[a][kk] = as_bf16x8(v);
        }
    }
}

__device__ __forceinline__ float max3(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }

// All k-step fragments of a staged 32-row sub-tile into distinct registers: the reads are issued together
// and the MFMAs run back to back, instead of one LDS round trip per k-step.
template <int D>
__device__ __forceinline__ void load_frags(bf16x8 (&fr)[D / 16], const unsigned char* lds, int row0, int lane) {
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) fr[kk] = Stage<D>::frag(lds, row0, kk, lane);
}
// acc = A.B over all k-steps; STREAM_IS_A: the streamed fragment is the A (row) operand.
template <int KS, bool STREAM_IS_A>
__device__ __forceinline__ f32x16 mma_tile(const bf16x8 (&stat)[KS], const bf16x8 (&fr)[KS]) {
    f32x16 acc = {0};
#pragma unroll
    for (int kk = 0; kk < KS; ++kk)
        acc = STREAM_IS_A ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[kk], stat[kk], acc, 0, 0, 0)
                          : __builtin_amdgcn_mfma_f32_32x32x16_bf16(stat[kk], fr[kk], acc, 0, 0, 0);
    return acc;
}
// ---- fused kernel: Q and K are read from HBM once -------------------------------------------------------
// One workgroup of WV wavefronts owns up to WV PAIRS of 32-query tiles of one (sequence, layer, head): tile i
// is paired with tile T-1-i, so that every pair -- and therefore every wavefront -- has the same amount of
// causal work (T+1 tile products per sweep).  With WV = 12 a head of up to 768 positions is ONE workgroup (one
// per CU, three wavefronts per SIMD: their MFMA chains and softmax phases overlap each other) and its keys pass
// through LDS exactly once per sweep.  The wavefront keeps its two query tiles in registers for the whole
// kernel and the keys stream through LDS (128-row stages, asynchronous copies, double-buffered) twice:
//   sweep 1:  S^T = K.Q^T (a lane holds one query): online max / sum -> lse of the wavefront's 64 rows
//   sweep 2:  S   = Q.K^T (a lane holds one key):   exp2(c*s - lse) summed over the lane's 32 query rows,
//             i.e. the column sums of this workgroup's rows; the keys come back from L2 / the last-level cache.
// Swapping the MFMA operands transposes the product, so the same stationary fragments serve both sweeps.  The
// column sums of one 128-key stage leave the workgroup once per stage: the wavefronts' values meet in LDS
// behind the barrier the stage needs anyway and are added in a fixed order (no atomics, bitwise reproducible).
// The workgroups of one head (long prompts) sit on one XCD next to each other in dispatch order and share the
// head's keys through that XCD's L2.
struct FusedParams {
    int B, L, H, Hkv, N, D;
    int T;                     // 32-row tiles: ceil(N / 32)
    int npairs;                // ceil(T / 2)
    int G;                     // workgroups per head: ceil(npairs / wavefronts per workgroup)
    long long nheads;          // B*L*H
    long long chunk;           // logical workgroup ids per XCD (a multiple of G)
    const bf16_t* q; Strides qs;
    const bf16_t* k; Strides ks;
    const float* scale;        // [L]
    const float* lse_in;       // [B,L,H,N] natural log, or unused
    float* partial;            // [B*L*H][G][N]: workgroup g's column sums of keys [0, min(N, 32*(T-4g)))
};

// barrier that orders LDS traffic only: loads from global memory that are still in flight stay in flight
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}
// one wavefront copies a whole stage (rolled loop: a few address registers)
template <int D>
__device__ __forceinline__ void copy_stage(const bf16_t* base, int64_t ld, int row0, int N, unsigned char* lds, int lane) {
    using S1 = Stage<D, 1>;
#pragma unroll 2
    for (int inst = 0; inst < S1::PIECES; ++inst) {
        const int L = inst * 64 + lane;
        const int row = L / S1::CPR, pos = L % S1::CPR;
        const int c = pos ^ ((row / S1::RPB) & (S1::CPR - 1));
        int grow = row0 + row;
        grow = grow < N ? grow : N - 1;
        const bf16_t* g = base + ((uint32_t)grow * (uint32_t)ld + (uint32_t)(c * 8));
        __builtin_amdgcn_global_load_lds((glb_void_t*)g, (lds_void_t*)(lds + inst * 1024), 16, 0, 0);
    }
}
template <int D>
__device__ __forceinline__ void load_stationary_one(bf16x8 (&f)[D / 16], const bf16_t* base, int64_t ld, int row0,
                                                    int N, int lane, bool flip) {
    const uint32_t sgn = flip ? 0x80008000u : 0u;
    int row = row0 + (lane & 31);
    row = row < N ? row : N - 1;
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) {
        uint4 v = *(const uint4*)(base + (int64_t)row * ld + 16 * kk + 8 * (lane >> 5));
        v.x ^= sgn; v.y ^= sgn; v.z ^= sgn; v.w ^= sgn;
        f[kk] = as_bf16x8(v);
    }
}

// WV wavefronts per workgroup; OCC wavefronts per SIMD the register allocation must allow.
// SPREAD (short prompts without a given lse, last wavefront without tiles): see the start of the kernel.
template <int D, bool HAS_LSE, int WV, int OCC, bool SPREAD>
__global__ void __launch_bounds__(WV * kWave, OCC)
importance_fused_kernel(FusedParams p) {
    static_assert(!(SPREAD && HAS_LSE), "the spread start belongs to the first sweep");
    constexpr int KS = D / 16;
    constexpr int NSUB = kStage / 32;
    using St = Stage<D, WV>;
    __shared__ __attribute__((aligned(16))) unsigned char s_tile0[St::BYTES];   // even steps
    __shared__ __attribute__((aligned(16))) unsigned char s_tile1[St::BYTES];   // odd steps
    __shared__ float s_red[2][WV][NSUB][32];              // column sums of a wavefront's rows:
                                                          // [parity][wavefront][sub-tile][key]
    __shared__ __attribute__((aligned(16))) float s_nl2[WV][2][32];   // -lse (log2 units) of a wavefront's two
                                                          // tiles by row; -inf for rows that do not exist
    // the wavefront index as a scalar: everything derived from it (which tiles exist, which sub-tiles are
    // needed) is then known to be uniform and branches on it are scalar branches
    const int lane = threadIdx.x & 63, wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const long long id = (long long)(blockIdx.x % kXcds) * p.chunk + blockIdx.x / kXcds;
    const int g = (int)(id % p.G);
    const long long head = id / p.G;
    if (head >= p.nheads) return;
    const int h = (int)(head % p.H), l = (int)((head / p.H) % p.L), b = (int)(head / ((long long)p.H * p.L));
    const bf16_t* qb = p.q + p.qs.b * b + p.qs.l * l + p.qs.h * h;
    const bf16_t* kb = p.k + p.ks.b * b + p.ks.l * l + p.ks.h * (h / (p.H / p.Hkv));
    float* part = p.partial + ((size_t)head * p.G + g) * p.N;
    float c = p.scale[l] * kLog2e;
    const bool flip = c < 0.f;
    c = fmaxf(fabsf(c), 1e-30f);                           // > 0, so that c * (-inf) of a masked entry stays -inf

    // this wavefront's pair: the early tile tE and the late tile tL (only tL for the middle tile of an odd T)
    const int pi = WV * g + wv;
    int tE = pi < p.npairs ? pi : -1, tL = pi < p.npairs ? p.T - 1 - pi : -1;
    if (tE == tL) tE = -1;
    const int qlo0 = 32 * tE, qlo1 = 32 * tL;             // negative: tile absent
    const int klim = min(p.N, 32 * (p.T - WV * g));       // keys this workgroup's rows can see
    const int S = (klim + kStage - 1) / kStage;           // key stages per sweep
    // Steps t = t0 .. 2S-1: step t works on key stage t mod S, sweep 1 for t < S and sweep 2 from S on, out of
    // s_tile{(t - t0) & 1}; the stage of step t+1 is copied into the other buffer meanwhile.
    const int t0 = HAS_LSE ? S : 0;

    // SPREAD: the first sweep walks the key stages downwards: the late tiles are needed first (the last stage by
    // the two latest tiles only), the early tiles not before the low stages, so the queries are requested late
    // tile first and arrive while the first stages are worked on, instead of all before the first product.
    // For that the key copies are issued by the last wavefront alone -- the launcher picks this form only when
    // that wavefront has no tiles (fewer pairs than wavefronts) -- and the barriers order LDS traffic only: a
    // wavefront's query loads then stay in flight across barriers.  (Measured: -2..3 % at 680 positions; with
    // every wavefront busy and several workgroups per head it loses, 80 against 73 ms at 8192 positions.)
    const bool copier = wv == WV - 1;
    bf16x8 bq[2][KS];
    if constexpr (SPREAD) {
        if (copier) copy_stage<D>(kb, p.ks.n, (S - 1) * kStage, p.N, s_tile0, lane);
        else {
            if (tL >= 0) load_stationary_one<D>(bq[1], qb, p.qs.n, qlo1, p.N, lane, flip);
            if (tE >= 0) load_stationary_one<D>(bq[0], qb, p.qs.n, qlo0, p.N, lane, flip);
        }
    } else {
        St::issue(kb, p.ks.n, 0, p.N, s_tile0, wv, lane);
        load_stationary<D>(bq, qb, p.qs.n, tE < 0 ? 0 : qlo0, tL < 0 ? 0 : qlo1, p.N, lane, flip);
    }
    float mrun[2] = {-INFINITY, -INFINITY}, srun[2] = {0.f, 0.f};
    if (HAS_LSE) {
        const float* lse = p.lse_in + (size_t)head * p.N;
        if (lane < 32) {
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                const int t = a == 0 ? tE : tL, m = 32 * t + lane;
                const float v = lse[min(max(m, 0), p.N - 1)];
                s_nl2[wv][a][lane] = (t >= 0 && m < p.N) ? -v * kLog2e : -INFINITY;   // rows >= N weigh 0
            }
        }
    }
    if constexpr (SPREAD) {
        if (copier) wait_async_copies();
        lds_barrier();
    } else {
        wait_async_copies();
        __syncthreads();
    }
    int par = 0;

    // sweep 1, one key stage: S^T = K.Q^T, a lane holds one query and 16 keys
    auto stage1 = [&](const unsigned char* cur, int s) {
#pragma unroll
        for (int j = 0; j < NSUB; ++j) {
            const int n0 = s * kStage + 32 * j;            // first key of the sub-tile
            const bool need0 = tE >= 0 && n0 <= qlo0 + 31;
            const bool need1 = tL >= 0 && n0 <= qlo1 + 31;
            if (!need1) continue;                          // tE < tL: need0 implies need1
            // the two products of the sub-tile one after the other (16 accumulator registers live at a time: the
            // other wavefronts of the SIMD fill the gaps of the single MFMA chain)
            bf16x8 fr[KS];
            load_frags<D>(fr, cur, 32 * j, lane);
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                if (a == 0 && !need0) continue;
                const f32x16 acc = mma_tile<KS, true>(bq[a], fr);
                const int qlo = a == 0 ? qlo0 : qlo1;
                float mnew, msafe, ps = 0.f;
                if (n0 + 31 <= qlo) {                      // every key of the sub-tile is visible to every query
                    float mx = max3(acc[0], acc[1], acc[2]);
#pragma unroll
                    for (int r = 3; r < 15; r += 2) mx = max3(mx, acc[r], acc[r + 1]);
                    mx = fmaxf(mx, acc[15]);
                    mnew = fmaxf(mrun[a], mx * c);
                    msafe = mnew;
#pragma unroll
                    for (int r = 0; r < 16; ++r) ps += __builtin_amdgcn_exp2f(fmaf(acc[r], c, -msafe));
                } else {                                   // the diagonal sub-tile: mask key > query
                    int q = lane & 31;
                    asm volatile("" : "+v"(q));            // keeps the compares out of loop-invariant registers
                    float mx = -INFINITY;
#pragma unroll
                    for (int r = 0; r < 16; ++r) mx = acc_row(r, lane) <= q ? fmaxf(mx, acc[r]) : mx;
                    mnew = fmaxf(mrun[a], mx * c);
                    msafe = mnew == -INFINITY ? 0.f : mnew;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float e = __builtin_amdgcn_exp2f(fmaf(acc[r], c, -msafe));
                        ps += acc_row(r, lane) <= q ? e : 0.f;
                    }
                }
                srun[a] = srun[a] * __builtin_amdgcn_exp2f(mrun[a] - msafe) + ps;
                mrun[a] = mnew;
            }
        }
    };
    // lse of the wavefront's rows: lanes l and l^32 hold the two key halves of the same query; sweep 2 reads
    // the result by accumulator row from a wavefront-private LDS row
    auto finish_lse = [&]() {
#pragma unroll
        for (int a = 0; a < 2; ++a) {
            const float mo = __shfl_xor(mrun[a], 32, kWave), so = __shfl_xor(srun[a], 32, kWave);
            const float M = fmaxf(mrun[a], mo);
            const float Ssum = srun[a] * __builtin_amdgcn_exp2f(mrun[a] - M) + so * __builtin_amdgcn_exp2f(mo - M);
            const int t = a == 0 ? tE : tL;
            if (lane < 32) s_nl2[wv][a][lane] = (t >= 0 && 32 * t + lane < p.N) ? -(M + __log2f(Ssum)) : -INFINITY;
        }
    };
    // sweep 2, one key stage: S = Q.K^T, a lane holds one key and 16 queries; the column sums of each product
    // go to the product's own LDS slot
    auto stage2 = [&](const unsigned char* cur, int s) {
#pragma unroll
        for (int j = 0; j < NSUB; ++j) {
            const int n0 = s * kStage + 32 * j;
            const bool need0 = tE >= 0 && n0 <= qlo0 + 31;
            const bool need1 = tL >= 0 && n0 <= qlo1 + 31;
            float ps0 = 0.f, ps1 = 0.f;
            if (need1) {
                bf16x8 fr[KS];
                load_frags<D>(fr, cur, 32 * j, lane);
#pragma unroll
                for (int a = 0; a < 2; ++a) {
                    if (a == 0 && !need0) continue;
                    // -lse of accumulator rows 8q + 4*(lane/32) + 0..3: requested before the MFMA chain, so that
                    // the LDS round trip is over when the chain is
                    const float4* src = (const float4*)&s_nl2[wv][a][4 * (lane >> 5)];
                    float nl[16];
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4) {
                        const float4 x = src[2 * q4];
                        nl[4 * q4] = x.x; nl[4 * q4 + 1] = x.y; nl[4 * q4 + 2] = x.z; nl[4 * q4 + 3] = x.w;
                    }
                    const f32x16 acc = mma_tile<KS, false>(bq[a], fr);
                    const int qlo = a == 0 ? qlo0 : qlo1;
                    float ps = 0.f;
                    if (n0 + 31 <= qlo) {                  // every key of the sub-tile is visible to every query
#pragma unroll
                        for (int r = 0; r < 16; ++r) ps += __builtin_amdgcn_exp2f(fmaf(acc[r], c, nl[r]));
                    } else {                               // the diagonal sub-tile: mask key > query
                        int key = lane & 31;
                        asm volatile("" : "+v"(key));      // keeps the compares out of loop-invariant registers
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const float pr = __builtin_amdgcn_exp2f(fmaf(acc[r], c, nl[r]));
                            ps += key <= acc_row(r, lane) ? pr : 0.f;
                        }
                    }
                    if (a == 0) ps0 = ps; else ps1 = ps;
                }
            }
            // lanes l and l+32 hold the two query halves of the same key
            const float ps = ps0 + ps1;
            const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(ps), __float_as_uint(ps), false, false);
            if (lane < 32) s_red[par][wv][j][lane] = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
        }
    };
    auto step = [&](const unsigned char* cur, unsigned char* nxt, int t) {
        if (t + 1 < 2 * S) St::issue(kb, p.ks.n, ((t + 1) % S) * kStage, p.N, nxt, wv, lane);
        const int s = t >= S ? t - S : t;
        if (t < S) {
            stage1(cur, s);
            if (t == S - 1) finish_lse();
            wait_async_copies();
            __syncthreads();
        } else {
            stage2(cur, s);
            wait_async_copies();
            __syncthreads();
            if (threadIdx.x < kStage) {
                const int sub = threadIdx.x >> 5, c32 = threadIdx.x & 31;
                float sum = 0.f;
#pragma unroll
                for (int w = 0; w < WV; ++w) sum += s_red[par][w][sub][c32];
                const int n = s * kStage + threadIdx.x;
                if (n < klim) part[n] = sum;
            }
            par ^= 1;
        }
    };
    if constexpr (!SPREAD) {
        for (int t = t0; t < 2 * S; t += 2) {
            step(s_tile0, s_tile1, t);
            if (t + 1 < 2 * S) step(s_tile1, s_tile0, t + 1);
        }
    } else {
        // step u of sweep 1 works on stage S-1-u, step u of sweep 2 on stage u; buffers alternate throughout
        auto flush = [&](int s) {
            if (threadIdx.x < kStage) {
                const int sub = threadIdx.x >> 5, c32 = threadIdx.x & 31;
                float sum = 0.f;
#pragma unroll
                for (int w = 0; w < WV; ++w) sum += s_red[par][w][sub][c32];
                const int n = s * kStage + threadIdx.x;
                if (n < klim) part[n] = sum;
            }
            par ^= 1;
        };
        auto step1 = [&](const unsigned char* cur, unsigned char* nxt, int u) {
            if (copier) copy_stage<D>(kb, p.ks.n, (u + 1 < S ? S - 2 - u : 0) * kStage, p.N, nxt, lane);
            stage1(cur, S - 1 - u);
            if (u == S - 1) finish_lse();
            if (copier) wait_async_copies();
            lds_barrier();
        };
        auto step2 = [&](const unsigned char* cur, unsigned char* nxt, int u) {
            if (copier && u + 1 < S) copy_stage<D>(kb, p.ks.n, (u + 1) * kStage, p.N, nxt, lane);
            stage2(cur, u);
            if (copier) wait_async_copies();
            lds_barrier();
            flush(u);
        };
        int sel = 0;
        for (int u = 0; u < S; ++u, sel ^= 1) {
            if (sel == 0) step1(s_tile0, s_tile1, u); else step1(s_tile1, s_tile0, u);
        }
        // every query load has been consumed by now; saying so keeps the second sweep free of waits for them
        __builtin_amdgcn_s_waitcnt(0x0F70);
        for (int u = 0; u < S; ++u, sel ^= 1) {
            if (sel == 0) step2(s_tile0, s_tile1, u); else step2(s_tile1, s_tile0, u);
        }
    }
}

// importance[b,l,n] = (1/H) * sum_h sum_g partial[b,l,h,g,n] over the workgroups g whose rows see key n.
// A workgroup takes 64 consecutive keys; its four wavefronts each add a quarter of the heads in (h, g) order
// (several loads in flight: the sum is bound by memory latency, not by bytes) and the four sums are added in
// wavefront order, so the result does not depend on timing.
constexpr int kMeanKeys = 64, kMeanParts = 4;
__global__ void __launch_bounds__(kMeanKeys * kMeanParts)
head_mean_fused_kernel(int H, int G, int N, int T, int WV, long long total, const float* __restrict__ partial,
                       float* __restrict__ importance) {
    __shared__ float s_acc[kMeanParts][kMeanKeys];
    const int lane = threadIdx.x % kMeanKeys, part = threadIdx.x / kMeanKeys;
    const long long i = (long long)blockIdx.x * kMeanKeys + lane;
    const bool live = i < total;
    const long long bl = live ? i / N : 0;
    const int n = live ? (int)(i % N) : 0;
    // workgroup g covers keys below 32*(T - WV*g): g <= (T - 1 - n/32) / WV
    const int gmax = min(G - 1, (T - 1 - n / 32) / WV);
    const int per = (H + kMeanParts - 1) / kMeanParts;
    const int h0 = part * per, h1 = min(H, h0 + per);
    const float* src = partial + (size_t)bl * H * G * N + n;
    float acc = 0.f;
    if (live) {
        if (G == 1) {
            int h = h0;
            for (; h + 8 <= h1; h += 8) {
                float v[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) v[j] = src[(size_t)(h + j) * N];
#pragma unroll
                for (int j = 0; j < 8; ++j) acc += v[j];
            }
            for (; h < h1; ++h) acc += src[(size_t)h * N];
        } else {
            for (int h = h0; h < h1; ++h) {
                const float* sh = src + (size_t)h * G * N;
                int g = 0;
                for (; g + 4 <= gmax + 1; g += 4) {
                    float v[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) v[j] = sh[(size_t)(g + j) * N];
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc += v[j];
                }
                for (; g <= gmax; ++g) acc += sh[(size_t)g * N];
            }
        }
    }
    s_acc[part][lane] = acc;
    __syncthreads();
    if (part == 0 && live) {
        float sum = s_acc[0][lane];
#pragma unroll
        for (int q = 1; q < kMeanParts; ++q) sum += s_acc[q][lane];
        importance[i] = sum / (float)H;
    }
}

// importance[b,l,n] = (1/H) * sum_h partial[b,l,h,n], heads added in order.
__global__ void head_mean_kernel(int H, int N, long long total, const float* __restrict__ partial,
                                 float* __restrict__ importance) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const long long bl = i / N;
    const int n = (int)(i % N);
    const float* src = partial + (size_t)bl * H * N + n;
    float acc = 0.f;
    int h = 0;
    for (; h + 8 <= H; h += 8) {             // eight loads in flight, added in head order
        float v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = src[(size_t)(h + j) * N];
#pragma unroll
        for (int j = 0; j < 8; ++j) acc += v[j];
    }
    for (; h < H; ++h) acc += src[(size_t)h * N];
    importance[i] = acc / (float)H;
}

// ---- plain kernels for fp32 storage -----------------------------------------------------------------
struct NaiveParams {
    int B, L, H, Hkv, N, D;
    const float* q; Strides qs;
    const float* k; Strides ks;
    const float* scale;
    const float* lse_in;
    float* lse_out;
    float* partial;
};

__global__ void lse_naive_kernel(NaiveParams p) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (long long)p.B * p.L * p.H * p.N) return;
    const int m = (int)(i % p.N);
    long long r = i / p.N;
    const int h = (int)(r % p.H); r /= p.H;
    const int l = (int)(r % p.L), b = (int)(r / p.L);
    const float* qr = p.q + p.qs.b * b + p.qs.l * l + p.qs.h * h + p.qs.n * m;
    const float* kb = p.k + p.ks.b * b + p.ks.l * l + p.ks.h * (h / (p.H / p.Hkv));
    const float c = p.scale[l] * kLog2e;
    float mrun = -INFINITY, srun = 0.f;
    for (int n = 0; n <= m; ++n) {
        const float* kr = kb + p.ks.n * n;
        float d = 0.f;
        for (int x = 0; x < p.D; ++x) d = fmaf(qr[x], kr[x], d);
        d *= c;
        const float mnew = fmaxf(mrun, d);
        srun = srun * exp2f(mrun - mnew) + exp2f(d - mnew);
        mrun = mnew;
    }
    p.lse_out[i] = (mrun + log2f(srun)) * kLn2;
}

__global__ void colsum_naive_kernel(NaiveParams p) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (long long)p.B * p.L * p.H * p.N) return;
    const int n = (int)(i % p.N);
    long long r = i / p.N;
    const int h = (int)(r % p.H); r /= p.H;
    const int l = (int)(r % p.L), b = (int)(r / p.L);
    const float* qb = p.q + p.qs.b * b + p.qs.l * l + p.qs.h * h;
    const float* kr = p.k + p.ks.b * b + p.ks.l * l + p.ks.h * (h / (p.H / p.Hkv)) + p.ks.n * n;
    const float* lse = p.lse_in + (i - n);
    const float c = p.scale[l] * kLog2e;
    float acc = 0.f;
    for (int m = n; m < p.N; ++m) {
        const float* qr = qb + p.qs.n * m;
        float d = 0.f;
        for (int x = 0; x < p.D; ++x) d = fmaf(qr[x], kr[x], d);
        acc += exp2f(d * c - lse[m] * kLog2e);
    }
    p.partial[i] = acc;
}

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// wavefronts per workgroup of the fused kernel: 12 (one workgroup per CU, three wavefronts per SIMD) so that a
// head of up to 768 positions is one workgroup and its keys pass through LDS once per sweep
constexpr int kFusedWaves = 12;
constexpr int kFusedOcc = 1;
static int fused_groups(int N) {
    const int T = (N + 31) / 32, npairs = (T + 1) / 2;
    return (npairs + kFusedWaves - 1) / kFusedWaves;
}

size_t importance_ws_bytes(const pkv_shape& s, bool has_lse) {
    const size_t per = align_up((size_t)s.B * s.L * s.H * s.N * sizeof(float), 256);
    if (s.dtype == PKV_F32) return per * (has_lse ? 1 : 2);
    // bf16: one row of column sums per (head, workgroup of the head)
    return align_up((size_t)s.B * s.L * s.H * fused_groups(s.N) * s.N * sizeof(float), 256);
}

hipError_t launch_importance(const pkv_shape& s, const void* q, Strides qs, const void* k, Strides ks,
                             const float* scale, const float* lse, float* importance, void* ws,
                             hipStream_t st) {
    const size_t per = align_up((size_t)s.B * s.L * s.H * s.N * sizeof(float), 256);
    float* partial = (float*)ws;
    const long long rows = (long long)s.B * s.L * s.H * s.N;
    const long long total = (long long)s.B * s.L * s.N;
    hipError_t e;
    if (s.dtype == PKV_F32) {
        float* lse_ws = (float*)((unsigned char*)ws + per);
        NaiveParams p{s.B, s.L, s.H, s.Hkv, s.N, s.D, (const float*)q, qs, (const float*)k, ks, scale,
                      lse ? lse : lse_ws, lse_ws, partial};
        const int nb = (int)((rows + 127) / 128);
        if (!lse) {
            hipLaunchKernelGGL(lse_naive_kernel, dim3(nb), dim3(128), 0, st, p);
            if ((e = hipGetLastError()) != hipSuccess) return e;
        }
        hipLaunchKernelGGL(colsum_naive_kernel, dim3(nb), dim3(128), 0, st, p);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        hipLaunchKernelGGL(head_mean_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, s.H, s.N,
                           total, partial, importance);
        return hipGetLastError();
    }
    FusedParams p;
    p.B = s.B; p.L = s.L; p.H = s.H; p.Hkv = s.Hkv; p.N = s.N; p.D = s.D;
    p.T = (s.N + 31) / 32;
    p.npairs = (p.T + 1) / 2;
    p.G = fused_groups(s.N);
    p.nheads = (long long)s.B * s.L * s.H;
    p.chunk = (p.nheads + kXcds - 1) / kXcds * p.G;          // whole heads per XCD
    p.q = (const bf16_t*)q; p.qs = qs; p.k = (const bf16_t*)k; p.ks = ks; p.scale = scale;
    p.lse_in = lse; p.partial = partial;
    const long long nblk = p.chunk * kXcds;
    if (nblk > 0x7fffffffll) return hipErrorInvalidValue;
    const dim3 grid((unsigned)nblk), block(kFusedWaves * kWave);
    const bool spread = !lse && p.G == 1 && p.npairs < kFusedWaves;   // the last wavefront only copies
    if (lse) {
        if (s.D == 128) hipLaunchKernelGGL((importance_fused_kernel<128, true, kFusedWaves, kFusedOcc, false>), grid, block, 0, st, p);
        else hipLaunchKernelGGL((importance_fused_kernel<64, true, kFusedWaves, kFusedOcc, false>), grid, block, 0, st, p);
    } else if (spread) {
        if (s.D == 128) hipLaunchKernelGGL((importance_fused_kernel<128, false, kFusedWaves, kFusedOcc, true>), grid, block, 0, st, p);
        else hipLaunchKernelGGL((importance_fused_kernel<64, false, kFusedWaves, kFusedOcc, true>), grid, block, 0, st, p);
    } else {
        if (s.D == 128) hipLaunchKernelGGL((importance_fused_kernel<128, false, kFusedWaves, kFusedOcc, false>), grid, block, 0, st, p);
        else hipLaunchKernelGGL((importance_fused_kernel<64, false, kFusedWaves, kFusedOcc, false>), grid, block, 0, st, p);
    }
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(head_mean_fused_kernel, dim3((unsigned)((total + kMeanKeys - 1) / kMeanKeys)),
                       dim3(kMeanKeys * kMeanParts), 0, st, s.H, p.G, s.N, p.T, kFusedWaves, total, partial, importance);
    return hipGetLastError();
}

}  // namespace pkv
