// Stage 1: KV importance (Sec. 3.2) -- column sums of the causal softmax, averaged over heads.
//
// bf16 inputs run on the matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulate) in two passes:
//
//  lse_mfma_kernel     query-stationary.  A wavefront keeps 32 query rows as the B operand in
//                      registers, key tiles stream through LDS (A operand), and an online max/sum per
//                      lane yields log sum_{j<=m} exp(scale*q_m.k_j) for every causal row m.
//  colsum_mfma_kernel  key-stationary.  A wavefront keeps 32 key rows as the A operand in registers,
//                      query tiles (and their lse) stream through LDS, and exp2(s*c - lse) is added
//                      into per-key accumulators in registers.  No atomics: the 32 query lanes of a
//                      key are summed through LDS in a fixed order at the end.
//
// Both compute S^T = K.Q^T so that a lane's 16 accumulator values belong to ONE query (column) and 16
// different keys (rows): the per-query quantity (running max / lse) is a scalar per lane.
// Only tiles on or below the diagonal are visited.  The head mean is a third, tiny kernel that adds
// the per-head partial sums in head order, so the result is bitwise reproducible.
//
// fp32 inputs (small validation shapes) use plain one-thread-per-row kernels with the same structure.
#include "pkv_common.hpp"

namespace pkv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr int kTile = 128;    // stationary rows per workgroup (4 wavefronts x 32)
constexpr int kStage = 64;    // streamed rows per LDS stage

struct ImpParams {
    int B, L, H, Hkv, N, D, ntiles;
    long long nwork;           // B*L*H*ntiles
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

// Copy `kStage` rows (row index clamped to N-1) of a [N, D] bf16 matrix with row stride `ld` elements
// into LDS with a padded row pitch; 256 threads, 16 bytes each per step.
template <int D>
__device__ __forceinline__ void stage_load(uint4* regs, const bf16_t* base, int64_t ld, int row0, int N) {
    constexpr int CPR = D / 8;                      // 16-byte chunks per row
    constexpr int PER = kStage * CPR / 256;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        const int id = threadIdx.x + 256 * j;
        int row = row0 + id / CPR;
        row = row < N ? row : N - 1;
        regs[j] = *(const uint4*)(base + (int64_t)row * ld + (id % CPR) * 8);
    }
}
template <int D>
__device__ __forceinline__ void stage_store(const uint4* regs, unsigned char* lds) {
    constexpr int CPR = D / 8;
    constexpr int PER = kStage * CPR / 256;
    constexpr int PITCH = D * 2 + 16;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        const int id = threadIdx.x + 256 * j;
        *(uint4*)(lds + (id / CPR) * PITCH + (id % CPR) * 16) = regs[j];
    }
}
// Operand fragment for k-step kk of the 32 rows starting at `row0` of a staged tile.
template <int D>
__device__ __forceinline__ bf16x8 lds_frag(const unsigned char* lds, int row0, int kk, int lane) {
    constexpr int PITCH = D * 2 + 16;
    return as_bf16x8(*(const uint4*)(lds + (row0 + (lane & 31)) * PITCH + (16 * kk + 8 * (lane >> 5)) * 2));
}

__device__ __forceinline__ void decode_work(const ImpParams& p, long long id, int& b, int& l, int& h, int& t) {
    t = (int)(id % p.ntiles); id /= p.ntiles;
    h = (int)(id % p.H); id /= p.H;
    l = (int)(id % p.L);
    b = (int)(id / p.L);
}

template <int D>
__global__ void __launch_bounds__(256)
lse_mfma_kernel(ImpParams p) {
    constexpr int KS = D / 16;
    constexpr int PITCH = D * 2 + 16;
    __shared__ __attribute__((aligned(16))) unsigned char s_tile[2][kStage * PITCH];
    const long long id = xcd_swizzle(blockIdx.x, gridDim.x);
    if (id >= p.nwork) return;
    int b, l, h, t;
    decode_work(p, id, b, l, h, t);
    t = p.ntiles - 1 - t;  // heavy (late) query tiles first
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int m0 = t * kTile, mw = m0 + 32 * wv;          // first query row of the workgroup / wavefront
    const bf16_t* qb = p.q + p.qs.b * b + p.qs.l * l + p.qs.h * h;
    const bf16_t* kb = p.k + p.ks.b * b + p.ks.l * l + p.ks.h * (h / (p.H / p.Hkv));
    const float c = p.scale[l] * kLog2e;

    bf16x8 bq[KS];
    {
        int row = mw + (lane & 31);
        row = row < p.N ? row : p.N - 1;
#pragma unroll
        for (int kk = 0; kk < KS; ++kk)
            bq[kk] = as_bf16x8(*(const uint4*)(qb + (int64_t)row * p.qs.n + 16 * kk + 8 * (lane >> 5)));
    }
    const int m = mw + (lane & 31);                        // this lane's query row
    const int nend = min(p.N, m0 + kTile);                 // keys needed by the workgroup: [0, nend)
    const int nstages = (nend + kStage - 1) / kStage;
    float mrun = -INFINITY, srun = 0.f;

    uint4 regs[kStage * (D / 8) / 256];
    stage_load<D>(regs, kb, p.ks.n, 0, p.N);
    stage_store<D>(regs, s_tile[0]);
    __syncthreads();
    for (int s = 0; s < nstages; ++s) {
        const unsigned char* cur = s_tile[s & 1];
        if (s + 1 < nstages) stage_load<D>(regs, kb, p.ks.n, (s + 1) * kStage, p.N);
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int n0 = s * kStage + 32 * half;          // first key of the 32x32 tile
            if (n0 > mw + 31 || mw >= p.N) continue;        // wavefront-uniform: above the diagonal / no rows
            f32x16 acc = {0};
#pragma unroll
            for (int kk = 0; kk < KS; ++kk)
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_frag<D>(cur, 32 * half, kk, lane), bq[kk], acc, 0, 0, 0);
            const bool diag = n0 + 31 > mw;                 // some (key, query) pairs of the tile are masked
            float tv[16], mx = -INFINITY;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int n = n0 + acc_row(r, lane);
                tv[r] = (diag && n > m) ? -INFINITY : acc[r] * c;
                mx = fmaxf(mx, tv[r]);
            }
            const float mnew = fmaxf(mrun, mx);
            const float msafe = mnew == -INFINITY ? 0.f : mnew;
            float ps = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) ps += __builtin_amdgcn_exp2f(tv[r] - msafe);
            srun = srun * __builtin_amdgcn_exp2f(mrun - msafe) + ps;
            mrun = mnew;
        }
        if (s + 1 < nstages) stage_store<D>(regs, s_tile[(s + 1) & 1]);
        __syncthreads();
    }
    // lanes l and l^32 hold the two halves of the keys of the same query
    const float mo = __shfl_xor(mrun, 32, kWave), so = __shfl_xor(srun, 32, kWave);
    const float M = fmaxf(mrun, mo);  // finite: key 0 is visible to every query
    const float S = srun * __builtin_amdgcn_exp2f(mrun - M) + so * __builtin_amdgcn_exp2f(mo - M);
    if (lane < 32 && m < p.N)
        p.lse_out[(((size_t)b * p.L + l) * p.H + h) * p.N + m] = (M + __log2f(S)) * kLn2;
}

template <int D>
__global__ void __launch_bounds__(256)
colsum_mfma_kernel(ImpParams p) {
    constexpr int KS = D / 16;
    constexpr int PITCH = D * 2 + 16;
    constexpr int TILE_BYTES = kStage * PITCH;
    // the staging buffers are reused for the final 4 x 32 x 33 float reduction (16.9 KB)
    constexpr int SMEM = 2 * TILE_BYTES > 4 * 32 * 33 * 4 ? 2 * TILE_BYTES : 4 * 32 * 33 * 4;
    __shared__ __attribute__((aligned(16))) unsigned char s_raw[SMEM];
    __shared__ float s_lse[2][kStage];
    const long long id = xcd_swizzle(blockIdx.x, gridDim.x);
    if (id >= p.nwork) return;
    int b, l, h, t;
    decode_work(p, id, b, l, h, t);  // key tile 0 sees every query: heaviest first
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int n0 = t * kTile, nw = n0 + 32 * wv;           // first key of the workgroup / wavefront
    const bf16_t* qb = p.q + p.qs.b * b + p.qs.l * l + p.qs.h * h;
    const bf16_t* kb = p.k + p.ks.b * b + p.ks.l * l + p.ks.h * (h / (p.H / p.Hkv));
    const float* lse = p.lse_in + (((size_t)b * p.L + l) * p.H + h) * p.N;
    const float c = p.scale[l] * kLog2e;

    bf16x8 ak[KS];
    {
        int row = nw + (lane & 31);
        row = row < p.N ? row : p.N - 1;
#pragma unroll
        for (int kk = 0; kk < KS; ++kk)
            ak[kk] = as_bf16x8(*(const uint4*)(kb + (int64_t)row * p.ks.n + 16 * kk + 8 * (lane >> 5)));
    }
    float col[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) col[r] = 0.f;

    const int s0 = n0 / kStage;                            // first query stage that can see key n0
    const int nstages = (p.N + kStage - 1) / kStage;
    uint4 regs[kStage * (D / 8) / 256];
    float lreg = 0.f;
    auto load_lse = [&](int s) {                           // rows >= N get +inf: their weight is exp2(-inf) = 0
        if (threadIdx.x < kStage) {
            const int mrow = s * kStage + threadIdx.x;
            lreg = mrow < p.N ? lse[mrow] * kLog2e : INFINITY;
        }
    };
    stage_load<D>(regs, qb, p.qs.n, s0 * kStage, p.N);
    load_lse(s0);
    stage_store<D>(regs, s_raw);
    if (threadIdx.x < kStage) s_lse[0][threadIdx.x] = lreg;
    __syncthreads();
    for (int s = s0; s < nstages; ++s) {
        const int buf = (s - s0) & 1;
        const unsigned char* cur = s_raw + buf * TILE_BYTES;
        if (s + 1 < nstages) { stage_load<D>(regs, qb, p.qs.n, (s + 1) * kStage, p.N); load_lse(s + 1); }
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int mt = s * kStage + 32 * half;          // first query of the 32x32 tile
            if (mt + 31 < nw || mt >= p.N || nw >= p.N) continue;  // above the diagonal / out of range
            f32x16 acc = {0};
#pragma unroll
            for (int kk = 0; kk < KS; ++kk)
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ak[kk], lds_frag<D>(cur, 32 * half, kk, lane), acc, 0, 0, 0);
            const float l2 = s_lse[buf][32 * half + (lane & 31)];
            const int m = mt + (lane & 31);
            const bool diag = mt < nw + 31;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int n = nw + acc_row(r, lane);
                const float pr = __builtin_amdgcn_exp2f(acc[r] * c - l2);
                col[r] += (diag && n > m) ? 0.f : pr;
            }
        }
        if (s + 1 < nstages) {
            stage_store<D>(regs, s_raw + (buf ^ 1) * TILE_BYTES);
            if (threadIdx.x < kStage) s_lse[buf ^ 1][threadIdx.x] = lreg;
        }
        __syncthreads();
    }
    // sum the 32 query lanes of every key through LDS, fixed order
    float* red = (float*)s_raw;
#pragma unroll
    for (int r = 0; r < 16; ++r) red[(wv * 32 + acc_row(r, lane)) * 33 + (lane & 31)] = col[r];
    __syncthreads();
    if (threadIdx.x < kTile) {
        const int n = n0 + threadIdx.x;
        float sum = 0.f;
#pragma unroll
        for (int j = 0; j < 32; ++j) sum += red[threadIdx.x * 33 + j];
        if (n < p.N) p.partial[(((size_t)b * p.L + l) * p.H + h) * p.N + n] = sum;
    }
}

// importance[b,l,n] = (1/H) * sum_h partial[b,l,h,n], heads added in order.
__global__ void head_mean_kernel(int H, int N, long long total, const float* __restrict__ partial,
                                 float* __restrict__ importance) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const long long bl = i / N;
    const int n = (int)(i % N);
    float acc = 0.f;
    for (int h = 0; h < H; ++h) acc += partial[((size_t)bl * H + h) * N + n];
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
        p.ntiles = (s.N + kTile - 1) / kTile;
        p.nwork = (long long)s.B * s.L * s.H * p.ntiles;
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
