// Stage 1: KV importance (Sec. 3.2) -- column sums of the causal softmax, averaged over heads.
//
// bf16 inputs run on the matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulate) in two passes:
//
//  lse_mfma_kernel     query-stationary.  A wavefront keeps 64 query rows (two MFMA tiles) as the B
//                      operand in registers, key tiles stream through LDS (A operand), and an online
//                      max/sum per lane yields log sum_{j<=m} exp(scale*q_m.k_j) for every causal row m.
//  colsum_mfma_kernel  key-stationary.  A wavefront keeps 64 key rows as the A operand in registers,
//                      query tiles (and their lse) stream through LDS, and exp2(s*c - lse) is added
//                      into per-key accumulators in registers.  No atomics: the query lanes of a key
//                      are summed through LDS in a fixed order when the block is finished.
//
// Both compute S^T = K.Q^T so that a lane's 16 accumulator values belong to ONE query (column) and 16
// different keys (rows): the per-query quantity (running max / lse) is a scalar per lane.
//
// Work decomposition.  One workgroup (4 wavefronts) owns one (sequence, layer, head) -- or an
// interleaved share of its blocks when there are few heads -- and walks its 256-row stationary blocks
// one after the other; for each block the other operand streams through LDS in stages of 128 rows,
// restricted to the causal side of the diagonal.  All (block, stage) steps of the workgroup form one
// flat sequence and the streamed tile of the next step is always in flight (global -> registers) while
// the current one is computed, also across block boundaries, so the start-up latency of a block is
// paid once per workgroup, not once per block.  Every LDS fragment read feeds two MFMAs.
//
// The head mean is a third, tiny kernel that adds the per-head partial sums in head order, so the
// result is bitwise reproducible.  fp32 inputs (small validation shapes) use plain kernels.
#include "pkv_common.hpp"

namespace pkv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr int kBlock = 256;   // stationary rows per block (4 wavefronts x 64)
constexpr int kStage = 128;   // streamed rows per LDS stage

struct ImpParams {
    int B, L, H, Hkv, N, D;
    int nblocks;               // ceil(N / kBlock)
    int nsplit;                // workgroups per head; workgroup `split` takes blocks split, split+nsplit, ...
    long long nwork;           // B*L*H*nsplit
    const bf16_t* q; Strides qs;
    const bf16_t* k; Strides ks;
    const float* scale;        // [L]
    const float* lse_in;       // [B,L,H,N] natural log (read by the column-sum pass)
    float* lse_out;            // [B,L,H,N] (written by the lse pass)
    float* partial;            // [B,L,H,N] per-head column sums
};

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

template <int D> struct Stage {
    static constexpr int CPR = D / 8;                 // 16-byte chunks per row
    static constexpr int ROWB = D * 2;                // bytes per row
    static constexpr int RPB = 256 / ROWB;            // rows per 256 bytes (one pass over the 64 banks)
    static constexpr int BYTES = kStage * ROWB;
    static constexpr int INSTS = BYTES / 1024 / 4;    // load instructions per wavefront (4 wavefronts)
    // Issue the asynchronous copy of rows [row0, row0 + kStage) (clamped to N-1) into `lds`.
    static __device__ __forceinline__ void issue(const bf16_t* base, int64_t ld, int row0, int N,
                                                 unsigned char* lds, int wv, int lane) {
#pragma unroll
        for (int i = 0; i < INSTS; ++i) {
            const int inst = wv * INSTS + i;          // which 1 KB piece of the tile
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
// two tiles that share the streamed fragments, interleaved so that consecutive MFMAs are independent
template <int KS, bool STREAM_IS_A>
__device__ __forceinline__ void mma_tile2(const bf16x8 (&stat0)[KS], const bf16x8 (&stat1)[KS],
                                          const bf16x8 (&fr)[KS], f32x16& acc0, f32x16& acc1) {
    acc0 = (f32x16){0}; acc1 = (f32x16){0};
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
        if constexpr (STREAM_IS_A) {
            acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[kk], stat0[kk], acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[kk], stat1[kk], acc1, 0, 0, 0);
        } else {
            acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(stat0[kk], fr[kk], acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(stat1[kk], fr[kk], acc1, 0, 0, 0);
        }
    }
}

// The flat (block, stage) walk of one workgroup.  LSE: block i streams keys of stages [0, ceil(min(N,
// 256(i+1))/128)); COLSUM: block i streams queries of stages [2i, ceil(N/128)).
template <bool COLSUM>
struct Walk {
    int N, nblocks, nsplit, blk, s, s_end;
    __device__ __forceinline__ int first_stage(int b) const { return COLSUM ? b * (kBlock / kStage) : 0; }
    __device__ __forceinline__ int end_stage(int b) const {
        const int rows = COLSUM ? N : min(N, (b + 1) * kBlock);
        return (rows + kStage - 1) / kStage;
    }
    __device__ __forceinline__ void start(int n, int nb, int ns, int split) {
        N = n; nblocks = nb; nsplit = ns; blk = split; s = first_stage(blk); s_end = end_stage(blk);
    }
    __device__ __forceinline__ bool last_stage_of_block() const { return s + 1 >= s_end; }
    __device__ __forceinline__ bool has_next_block() const { return blk + nsplit < nblocks; }
    // the step after the current one (the current one again if it is the very last)
    __device__ __forceinline__ void peek(int& nb, int& ns) const {
        if (!last_stage_of_block()) { nb = blk; ns = s + 1; }
        else if (has_next_block()) { nb = blk + nsplit; ns = first_stage(nb); }
        else { nb = blk; ns = s; }
    }
    __device__ __forceinline__ void advance() {
        if (!last_stage_of_block()) { ++s; }
        else { blk += nsplit; s = first_stage(blk); s_end = end_stage(blk); }
    }
};

__device__ __forceinline__ void decode_work(const ImpParams& p, long long id, int& b, int& l, int& h, int& split) {
    split = (int)(id % p.nsplit); id /= p.nsplit;
    h = (int)(id % p.H); id /= p.H;
    l = (int)(id % p.L);
    b = (int)(id / p.L);
}

template <int D>
__global__ void __launch_bounds__(256, 2)
lse_mfma_kernel(ImpParams p) {
    constexpr int KS = D / 16;
    using St = Stage<D>;
    // two staging buffers as separate objects: the compiler can then tell that the copy in flight into one
    // does not alias the fragment reads from the other, and does not wait for it
    __shared__ __attribute__((aligned(16))) unsigned char s_tileA[St::BYTES];
    __shared__ __attribute__((aligned(16))) unsigned char s_tileB[St::BYTES];
    const long long id = xcd_swizzle(blockIdx.x, gridDim.x);
    if (id >= p.nwork) return;
    int b, l, h, split;
    decode_work(p, id, b, l, h, split);
    if (split >= p.nblocks) return;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const bf16_t* qb = p.q + p.qs.b * b + p.qs.l * l + p.qs.h * h;
    const bf16_t* kb = p.k + p.ks.b * b + p.ks.l * l + p.ks.h * (h / (p.H / p.Hkv));
    float* lse_row = p.lse_out + (((size_t)b * p.L + l) * p.H + h) * p.N;
    float c = p.scale[l] * kLog2e;
    const bool flip = c < 0.f;
    c = fabsf(c);

    Walk<false> w;
    w.start(p.N, p.nblocks, p.nsplit, split);
    St::issue(kb, p.ks.n, w.s * kStage, p.N, s_tileA, wv, lane);
    // Wavefront w owns the 32-row tiles w and 7-w of the block: an early and a late tile, so that the causal
    // triangle gives every wavefront of a diagonal block the same amount of work.
    bf16x8 bq[2][KS];
    int qlo0 = w.blk * kBlock + 32 * wv, qlo1 = w.blk * kBlock + 32 * (7 - wv);
    load_stationary<D>(bq, qb, p.qs.n, qlo0, qlo1, p.N, lane, flip);
    float mrun[2] = {-INFINITY, -INFINITY}, srun[2] = {0.f, 0.f};
    wait_async_copies();
    __syncthreads();

    // one (block, stage) step: compute from `cur` while the next step's keys are copied into `nxt`;
    // returns true after the last step
    auto step = [&](const unsigned char* cur, unsigned char* nxt) -> bool {
        int nb, ns;
        w.peek(nb, ns);
        St::issue(kb, p.ks.n, ns * kStage, p.N, nxt, wv, lane);   // (this step's keys again at the very end)
#pragma unroll
        for (int j = 0; j < kStage / 32; ++j) {
            const int n0 = w.s * kStage + 32 * j;          // first key of the sub-tile
            // tile a holds queries [qlo_a, qlo_a+31]; needed unless all keys of the sub-tile lie above the diagonal
            const bool need0 = n0 <= qlo0 + 31 && qlo0 < p.N && n0 < p.N;
            const bool need1 = n0 <= qlo1 + 31 && qlo1 < p.N && n0 < p.N;
            if (!(need0 || need1)) continue;
            f32x16 acc0 = {0}, acc1 = {0};
            bf16x8 fr[KS];
            load_frags<D>(fr, cur, 32 * j, lane);
            if (need0 && need1) mma_tile2<KS, true>(bq[0], bq[1], fr, acc0, acc1);
            else if (need0) acc0 = mma_tile<KS, true>(bq[0], fr);
            else acc1 = mma_tile<KS, true>(bq[1], fr);
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                if (!(a == 0 ? need0 : need1)) continue;
                const f32x16 acc = a == 0 ? acc0 : acc1;
                const int qlo = a == 0 ? qlo0 : qlo1;
                float mnew, msafe, ps = 0.f;
                if (n0 + 31 <= qlo) {                      // every key of the sub-tile is visible to every query
                    float mx = max3(acc[0], acc[1], acc[2]);
#pragma unroll
                    for (int r = 3; r < 15; r += 2) mx = max3(mx, acc[r], acc[r + 1]);
                    mx = fmaxf(mx, acc[15]);
                    mnew = fmaxf(mrun[a], mx * c);
                    msafe = mnew;                          // finite: it covers 16 visible keys
#pragma unroll
                    for (int r = 0; r < 16; ++r) ps += __builtin_amdgcn_exp2f(fmaf(acc[r], c, -msafe));
                } else {                                   // the sub-tile touches the diagonal: mask key > query
                    const int dm = qlo + (lane & 31) - n0; // key row i of the sub-tile is visible iff i <= dm
                    float mx = -INFINITY;
#pragma unroll
                    for (int r = 0; r < 16; ++r) mx = acc_row(r, lane) <= dm ? fmaxf(mx, acc[r]) : mx;
                    mnew = fmaxf(mrun[a], mx * c);
                    msafe = mnew == -INFINITY ? 0.f : mnew;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float e = __builtin_amdgcn_exp2f(fmaf(acc[r], c, -msafe));
                        ps += acc_row(r, lane) <= dm ? e : 0.f;
                    }
                }
                srun[a] = srun[a] * __builtin_amdgcn_exp2f(mrun[a] - msafe) + ps;
                mrun[a] = mnew;
            }
        }
        wait_async_copies();
        __syncthreads();
        if (w.last_stage_of_block()) {
            // lanes l and l^32 hold the two key halves of the same query
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                const float mo = __shfl_xor(mrun[a], 32, kWave), so = __shfl_xor(srun[a], 32, kWave);
                const float M = fmaxf(mrun[a], mo);        // finite for m < N: key 0 is visible to every query
                const float S = srun[a] * __builtin_amdgcn_exp2f(mrun[a] - M) + so * __builtin_amdgcn_exp2f(mo - M);
                const int m = (a == 0 ? qlo0 : qlo1) + lane;
                if (lane < 32 && m < p.N) lse_row[m] = (M + __log2f(S)) * kLn2;
                mrun[a] = -INFINITY; srun[a] = 0.f;
            }
            if (!w.has_next_block()) return true;
            qlo0 = (w.blk + w.nsplit) * kBlock + 32 * wv;
            qlo1 = (w.blk + w.nsplit) * kBlock + 32 * (7 - wv);
            load_stationary<D>(bq, qb, p.qs.n, qlo0, qlo1, p.N, lane, flip);
        }
        w.advance();
        return false;
    };
    while (true) {
        if (step(s_tileA, s_tileB)) break;
        if (step(s_tileB, s_tileA)) break;
    }
}

template <int D>
__global__ void __launch_bounds__(256, 2)
colsum_mfma_kernel(ImpParams p) {
    constexpr int KS = D / 16;
    using St = Stage<D>;
    constexpr int RED_BYTES = 4 * 64 * 33 * 4;             // wavefront x 64 keys x 32 query lanes (+1 pad)
    constexpr int BUF = St::BYTES > RED_BYTES ? St::BYTES : RED_BYTES;   // a consumed staging buffer doubles as
                                                                          // the reduction buffer
    // separate objects, so that the copy in flight into one buffer is known not to alias reads of the other
    __shared__ __attribute__((aligned(16))) unsigned char s_tileA[BUF];
    __shared__ __attribute__((aligned(16))) unsigned char s_tileB[BUF];
    __shared__ __attribute__((aligned(16))) float s_lseA[kStage];
    __shared__ __attribute__((aligned(16))) float s_lseB[kStage];
    const long long id = xcd_swizzle(blockIdx.x, gridDim.x);
    if (id >= p.nwork) return;
    int b, l, h, split;
    decode_work(p, id, b, l, h, split);
    if (split >= p.nblocks) return;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const bf16_t* qb = p.q + p.qs.b * b + p.qs.l * l + p.qs.h * h;
    const bf16_t* kb = p.k + p.ks.b * b + p.ks.l * l + p.ks.h * (h / (p.H / p.Hkv));
    const float* lse = p.lse_in + (((size_t)b * p.L + l) * p.H + h) * p.N;
    float* part_row = p.partial + (((size_t)b * p.L + l) * p.H + h) * p.N;
    float c = p.scale[l] * kLog2e;
    const bool flip = c < 0.f;
    c = fabsf(c);
    Walk<true> w;
    w.start(p.N, p.nblocks, p.nsplit, split);
    // the lse of the staged query rows travels the same way: 4-byte copies, lane i -> dst[64*wv + i]
    auto issue_lse = [&](int stage, float* dst) {
        if (wv < kStage / 64) {
            int mrow = stage * kStage + 64 * wv + lane;
            mrow = mrow < p.N ? mrow : p.N - 1;
            __builtin_amdgcn_global_load_lds((glb_void_t*)(lse + mrow), (lds_void_t*)(dst + 64 * wv), 4, 0, 0);
        }
    };
    St::issue(qb, p.qs.n, w.s * kStage, p.N, s_tileA, wv, lane);
    issue_lse(w.s, s_lseA);
    // Wavefront w owns the 32-row key tiles w and 7-w of the block (balanced causal work, as in the lse pass).
    bf16x8 ak[2][KS];
    int klo0 = w.blk * kBlock + 32 * wv, klo1 = w.blk * kBlock + 32 * (7 - wv);
    load_stationary<D>(ak, kb, p.ks.n, klo0, klo1, p.N, lane, flip);
    float col[2][16];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int r = 0; r < 16; ++r) col[a][r] = 0.f;
    wait_async_copies();
    __syncthreads();

    // one (block, stage) step: compute from `cur` while the next step's queries and lse are copied into `nxt`;
    // returns true after the last step
    auto step = [&](unsigned char* cur, const float* cur_lse, unsigned char* nxt, float* nxt_lse) -> bool {
        int nb, ns;
        w.peek(nb, ns);
        St::issue(qb, p.qs.n, ns * kStage, p.N, nxt, wv, lane);   // (this step's rows again at the very end)
        issue_lse(ns, nxt_lse);
#pragma unroll
        for (int j = 0; j < kStage / 32; ++j) {
            const int mt = w.s * kStage + 32 * j;          // first query of the sub-tile
            // tile a holds keys [klo_a, klo_a+31]; needed unless all queries of the sub-tile lie before its keys
            const bool need0 = mt + 31 >= klo0 && klo0 < p.N && mt < p.N;
            const bool need1 = mt + 31 >= klo1 && klo1 < p.N && mt < p.N;
            if (!need0) continue;                          // klo0 <= klo1: need1 implies need0
            f32x16 acc0 = {0}, acc1 = {0};
            bf16x8 fr[KS];
            load_frags<D>(fr, cur, 32 * j, lane);
            if (need1) mma_tile2<KS, false>(ak[0], ak[1], fr, acc0, acc1);
            else acc0 = mma_tile<KS, false>(ak[0], fr);
            const int m = mt + (lane & 31);
            // rows >= N carry +inf: their weight is exp2(-inf) = 0
            const float l2 = m < p.N ? cur_lse[32 * j + (lane & 31)] * kLog2e : INFINITY;
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                if (a == 1 && !need1) continue;
                const f32x16 acc = a == 0 ? acc0 : acc1;
                const int klo = a == 0 ? klo0 : klo1;
                if (mt >= klo + 31) {                      // every query of the sub-tile sees every key of the tile
#pragma unroll
                    for (int r = 0; r < 16; ++r) col[a][r] += __builtin_amdgcn_exp2f(fmaf(acc[r], c, -l2));
                } else {
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float pr = __builtin_amdgcn_exp2f(fmaf(acc[r], c, -l2));
                        col[a][r] += (klo + acc_row(r, lane) > m) ? 0.f : pr;
                    }
                }
            }
        }
        wait_async_copies();
        __syncthreads();
        if (w.last_stage_of_block()) {
            // The block is complete.  Fetch the next block's keys first (independent of the reduction), then
            // sum the 32 query lanes of every key through the staging buffer that was just consumed.
            const bool more = w.has_next_block();
            const int kold0 = klo0, kold1 = klo1;
            if (more) {
                klo0 = (w.blk + w.nsplit) * kBlock + 32 * wv;
                klo1 = (w.blk + w.nsplit) * kBlock + 32 * (7 - wv);
                load_stationary<D>(ak, kb, p.ks.n, klo0, klo1, p.N, lane, flip);
            }
            float* red = (float*)cur + wv * 64 * 33;
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    red[(32 * a + acc_row(r, lane)) * 33 + (lane & 31)] = col[a][r];
                    col[a][r] = 0.f;
                }
            __syncthreads();
            {
                float sum = 0.f;
#pragma unroll
                for (int j = 0; j < 32; ++j) sum += red[lane * 33 + j];
                const int n = (lane < 32 ? kold0 : kold1 - 32) + lane;   // red rows 0..31 = tile 0, 32..63 = tile 1
                if (n < p.N) part_row[n] = sum;
            }
            __syncthreads();                               // `cur` becomes a copy target in the next step
            if (!more) return true;
        }
        w.advance();
        return false;
    };
    while (true) {
        if (step(s_tileA, s_lseA, s_tileB, s_lseB)) break;
        if (step(s_tileB, s_lseB, s_tileA, s_lseA)) break;
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

size_t importance_ws_bytes(const pkv_shape& s, bool has_lse) {
    const size_t per = align_up((size_t)s.B * s.L * s.H * s.N * sizeof(float), 256);
    return per * (has_lse ? 1 : 2);
}

hipError_t launch_importance(const pkv_shape& s, const void* q, Strides qs, const void* k, Strides ks,
                             const float* scale, const float* lse, float* importance, void* ws,
                             hipStream_t st) {
    const size_t per = align_up((size_t)s.B * s.L * s.H * s.N * sizeof(float), 256);
    float* partial = (float*)ws;
    float* lse_ws = (float*)((unsigned char*)ws + per);
    const long long rows = (long long)s.B * s.L * s.H * s.N;
    hipError_t e;
    if (s.dtype == PKV_F32) {
        NaiveParams p{s.B, s.L, s.H, s.Hkv, s.N, s.D, (const float*)q, qs, (const float*)k, ks, scale,
                      lse ? lse : lse_ws, lse_ws, partial};
        const int nb = (int)((rows + 127) / 128);
        if (!lse) {
            hipLaunchKernelGGL(lse_naive_kernel, dim3(nb), dim3(128), 0, st, p);
            if ((e = hipGetLastError()) != hipSuccess) return e;
        }
        hipLaunchKernelGGL(colsum_naive_kernel, dim3(nb), dim3(128), 0, st, p);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    } else {
        ImpParams p;
        p.B = s.B; p.L = s.L; p.H = s.H; p.Hkv = s.Hkv; p.N = s.N; p.D = s.D;
        p.nblocks = (s.N + kBlock - 1) / kBlock;
        // one workgroup per head; with few heads, split a head's blocks over several workgroups
        const long long heads = (long long)s.B * s.L * s.H;
        long long want = (1024 + heads - 1) / heads;
        p.nsplit = (int)(want < 1 ? 1 : (want > p.nblocks ? p.nblocks : want));
        p.nwork = heads * p.nsplit;
        p.q = (const bf16_t*)q; p.qs = qs; p.k = (const bf16_t*)k; p.ks = ks; p.scale = scale;
        p.lse_in = lse ? lse : lse_ws; p.lse_out = lse_ws; p.partial = partial;
        const unsigned nblk = (unsigned)((p.nwork + kXcds - 1) / kXcds * kXcds);
        if (!lse) {
            if (s.D == 128) hipLaunchKernelGGL(lse_mfma_kernel<128>, dim3(nblk), dim3(256), 0, st, p);
            else hipLaunchKernelGGL(lse_mfma_kernel<64>, dim3(nblk), dim3(256), 0, st, p);
            if ((e = hipGetLastError()) != hipSuccess) return e;
        }
        if (s.D == 128) hipLaunchKernelGGL(colsum_mfma_kernel<128>, dim3(nblk), dim3(256), 0, st, p);
        else hipLaunchKernelGGL(colsum_mfma_kernel<64>, dim3(nblk), dim3(256), 0, st, p);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    const long long total = (long long)s.B * s.L * s.N;
    hipLaunchKernelGGL(head_mean_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, s.H, s.N,
                       total, partial, importance);
    return hipGetLastError();
}

}  // namespace pkv
