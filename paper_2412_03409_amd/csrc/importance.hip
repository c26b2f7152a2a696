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
//                      are summed through LDS in a fixed order at the end.
// In both, one LDS fragment read feeds two MFMAs (LDS bandwidth would otherwise cap the matrix cores),
// and two wavefronts share each stationary block, taking alternate halves of every streamed stage.
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

// ---- staging of a streamed 64-row tile: global -> registers -> padded LDS -----------------------------
// 256 threads move kStage rows of D bf16 (row index clamped to N-1) in 16-byte pieces.
template <int D> struct Stage {
    static constexpr int CPR = D / 8;                 // 16-byte chunks per row
    static constexpr int PER = kStage * CPR / 256;    // chunks per thread
    static constexpr int PITCH = D * 2 + 16;          // padded row pitch: conflict-free 16-byte reads
    static constexpr int BYTES = kStage * PITCH;
    uint4 r[PER];
    __device__ __forceinline__ void load(const bf16_t* base, int64_t ld, int row0, int N) {
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const int id = threadIdx.x + 256 * j;
            int row = row0 + id / CPR;
            row = row < N ? row : N - 1;
            r[j] = *(const uint4*)(base + (int64_t)row * ld + (id % CPR) * 8);
        }
    }
    __device__ __forceinline__ void store(unsigned char* lds) const {
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const int id = threadIdx.x + 256 * j;
            *(uint4*)(lds + (id / CPR) * PITCH + (id % CPR) * 16) = r[j];
        }
    }
    // MFMA operand fragment for k-step kk of the 32 rows starting at row0 of a staged tile
    static __device__ __forceinline__ bf16x8 frag(const unsigned char* lds, int row0, int kk, int lane) {
        return as_bf16x8(*(const uint4*)(lds + (row0 + (lane & 31)) * PITCH + (16 * kk + 8 * (lane >> 5)) * 2));
    }
};

// The wavefront's stationary operand: two tiles of 32 rows, straight from global memory into the MFMA
// register layout.  flip = the rows are negated (exact in bf16) so that the logit scale is positive.
template <int D>
__device__ __forceinline__ void load_stationary(bf16x8 (&f)[2][D / 16], const bf16_t* base, int64_t ld, int row0,
                                                int N, int lane, bool flip) {
#pragma unroll
    for (int a = 0; a < 2; ++a) {
        int row = row0 + 32 * a + (lane & 31);
        row = row < N ? row : N - 1;
#pragma unroll
        for (int kk = 0; kk < D / 16; ++kk) {
            uint4 v = *(const uint4*)(base + (int64_t)row * ld + 16 * kk + 8 * (lane >> 5));
            if (flip) { v.x ^= 0x80008000u; v.y ^= 0x80008000u; v.z ^= 0x80008000u; v.w ^= 0x80008000u; }
            f[a][kk] = as_bf16x8(v);
        }
    }
}

__device__ __forceinline__ void decode_work(const ImpParams& p, long long id, int& b, int& l, int& h, int& t) {
    t = (int)(id % p.ntiles); id /= p.ntiles;
    h = (int)(id % p.H); id /= p.H;
    l = (int)(id % p.L);
    b = (int)(id / p.L);
}

__device__ __forceinline__ float max3(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }

// Workgroup = 4 wavefronts = (row group g, parity par).  It owns 128 stationary rows (64 per group, two
// 32-row MFMA tiles per wavefront); the streamed operand arrives in stages of 64 rows and the wavefront
// of parity par takes the 32-row half `par`, so one LDS fragment read feeds two MFMAs.
template <int D>
__global__ void __launch_bounds__(256, 2)
lse_mfma_kernel(ImpParams p) {
    constexpr int KS = D / 16;
    using St = Stage<D>;
    __shared__ __attribute__((aligned(16))) unsigned char s_tile[2][St::BYTES];
    __shared__ float s_m[2][kTile], s_s[2][kTile];
    const long long id = xcd_swizzle(blockIdx.x, gridDim.x);
    if (id >= p.nwork) return;
    int b, l, h, t;
    decode_work(p, id, b, l, h, t);
    t = p.ntiles - 1 - t;  // heavy (late) query tiles first
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int g = wv >> 1, par = wv & 1;
    const int m0 = t * kTile, mq0 = m0 + 64 * g;           // first query of the workgroup / wavefront
    const bf16_t* qb = p.q + p.qs.b * b + p.qs.l * l + p.qs.h * h;
    const bf16_t* kb = p.k + p.ks.b * b + p.ks.l * l + p.ks.h * (h / (p.H / p.Hkv));
    float c = p.scale[l] * kLog2e;
    const bool flip = c < 0.f;
    c = fabsf(c);

    bf16x8 bq[2][KS];
    load_stationary<D>(bq, qb, p.qs.n, mq0, p.N, lane, flip);
    const int nend = min(p.N, m0 + kTile);                 // keys needed by the workgroup: [0, nend)
    const int nstages = (nend + kStage - 1) / kStage;
    float mrun[2] = {-INFINITY, -INFINITY}, srun[2] = {0.f, 0.f};

    St st;
    st.load(kb, p.ks.n, 0, p.N);
    st.store(s_tile[0]);
    __syncthreads();
    for (int s = 0; s < nstages; ++s) {
        const unsigned char* cur = s_tile[s & 1];
        st.load(kb, p.ks.n, (s + 1) * kStage, p.N);   // rows are clamped: the extra load after the last stage is harmless
        const int n0 = s * kStage + 32 * par;              // first key of this wavefront's half
        // tile a holds queries [mq0+32a, mq0+32a+31]; it is needed unless all its keys lie above the diagonal
        const bool need0 = n0 <= mq0 + 31 && mq0 < p.N;
        const bool need1 = n0 <= mq0 + 63 && mq0 + 32 < p.N;
        if (need0 || need1) {
            f32x16 acc0 = {0}, acc1 = {0};
#pragma unroll
            for (int kk = 0; kk < KS; ++kk) {
                const bf16x8 ka = St::frag(cur, 32 * par, kk, lane);
                if (need0) acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, bq[0][kk], acc0, 0, 0, 0);
                if (need1) acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, bq[1][kk], acc1, 0, 0, 0);
            }
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                if (!(a == 0 ? need0 : need1)) continue;
                f32x16 acc = a == 0 ? acc0 : acc1;
                const int qlo = mq0 + 32 * a;
                if (n0 + 31 > qlo) {                       // tile touches the diagonal: mask key > query
                    const int m = qlo + (lane & 31);
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (n0 + acc_row(r, lane) > m) acc[r] = -INFINITY;
                }
                float mx = max3(acc[0], acc[1], acc[2]);
#pragma unroll
                for (int r = 3; r < 15; r += 2) mx = max3(mx, acc[r], acc[r + 1]);
                mx = fmaxf(mx, acc[15]);
                const float mnew = fmaxf(mrun[a], mx * c);
                const float msafe = mnew == -INFINITY ? 0.f : mnew;
                float ps = 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) ps += __builtin_amdgcn_exp2f(fmaf(acc[r], c, -msafe));
                srun[a] = srun[a] * __builtin_amdgcn_exp2f(mrun[a] - msafe) + ps;
                mrun[a] = mnew;
            }
        }
        st.store(s_tile[(s + 1) & 1]);
        __syncthreads();
    }
    // lanes l and l^32 hold the two key halves of the same query; then the two parities merge via LDS
#pragma unroll
    for (int a = 0; a < 2; ++a) {
        const float mo = __shfl_xor(mrun[a], 32, kWave), so = __shfl_xor(srun[a], 32, kWave);
        const float M = fmaxf(mrun[a], mo);
        const float Ms = M == -INFINITY ? 0.f : M;
        const float S = srun[a] * __builtin_amdgcn_exp2f(mrun[a] - Ms) + so * __builtin_amdgcn_exp2f(mo - Ms);
        if (lane < 32) { s_m[par][64 * g + 32 * a + lane] = M; s_s[par][64 * g + 32 * a + lane] = S; }
    }
    __syncthreads();
    if (threadIdx.x < kTile) {
        const int m = m0 + threadIdx.x;
        const float ma = s_m[0][threadIdx.x], mb = s_m[1][threadIdx.x];
        const float M = fmaxf(ma, mb);                     // finite for m < N: key 0 is visible to every query
        const float S = s_s[0][threadIdx.x] * __builtin_amdgcn_exp2f(ma - M) +
                        s_s[1][threadIdx.x] * __builtin_amdgcn_exp2f(mb - M);
        if (m < p.N) p.lse_out[(((size_t)b * p.L + l) * p.H + h) * p.N + m] = (M + __log2f(S)) * kLn2;
    }
}

template <int D>
__global__ void __launch_bounds__(256, 2)
colsum_mfma_kernel(ImpParams p) {
    constexpr int KS = D / 16;
    using St = Stage<D>;
    constexpr int RED_BYTES = 4 * 64 * 33 * 4;             // (group, parity) x 64 keys x 32 query lanes (+1 pad)
    constexpr int SMEM = 2 * St::BYTES > RED_BYTES ? 2 * St::BYTES : RED_BYTES;
    __shared__ __attribute__((aligned(16))) unsigned char s_raw[SMEM];
    __shared__ float s_lse[2][kStage];
    const long long id = xcd_swizzle(blockIdx.x, gridDim.x);
    if (id >= p.nwork) return;
    int b, l, h, t;
    decode_work(p, id, b, l, h, t);                        // key tile 0 sees every query: heaviest first
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int g = wv >> 1, par = wv & 1;
    const int n0 = t * kTile, nk0 = n0 + 64 * g;           // first key of the workgroup / wavefront
    const bf16_t* qb = p.q + p.qs.b * b + p.qs.l * l + p.qs.h * h;
    const bf16_t* kb = p.k + p.ks.b * b + p.ks.l * l + p.ks.h * (h / (p.H / p.Hkv));
    const float* lse = p.lse_in + (((size_t)b * p.L + l) * p.H + h) * p.N;
    float c = p.scale[l] * kLog2e;
    const bool flip = c < 0.f;
    c = fabsf(c);

    bf16x8 ak[2][KS];
    load_stationary<D>(ak, kb, p.ks.n, nk0, p.N, lane, flip);
    float col[2][16];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int r = 0; r < 16; ++r) col[a][r] = 0.f;

    const int s0 = n0 / kStage;                            // first query stage that can see key n0
    const int nstages = (p.N + kStage - 1) / kStage;
    St st;
    float lreg = 0.f;
    st.load(qb, p.qs.n, s0 * kStage, p.N);
    if (threadIdx.x < kStage) {                            // rows >= N get +inf: their weight is exp2(-inf) = 0
        const int mrow = s0 * kStage + threadIdx.x;
        lreg = mrow < p.N ? lse[mrow] * kLog2e : INFINITY;
    }
    st.store(s_raw);
    if (threadIdx.x < kStage) s_lse[0][threadIdx.x] = lreg;
    __syncthreads();
    for (int s = s0; s < nstages; ++s) {
        const int buf = (s - s0) & 1;
        const unsigned char* cur = s_raw + buf * St::BYTES;
        st.load(qb, p.qs.n, (s + 1) * kStage, p.N);        // rows are clamped: harmless after the last stage
        if (threadIdx.x < kStage) {
            const int mrow = (s + 1) * kStage + threadIdx.x;
            lreg = mrow < p.N ? lse[mrow] * kLog2e : INFINITY;
        }
        const int mt = s * kStage + 32 * par;              // first query of this wavefront's half
        // tile a holds keys [nk0+32a, nk0+32a+31]; needed unless all its queries lie before all its keys
        const bool need0 = mt + 31 >= nk0 && nk0 < p.N && mt < p.N;
        const bool need1 = mt + 31 >= nk0 + 32 && nk0 + 32 < p.N && mt < p.N;
        if (need0) {                                       // need1 implies need0
            f32x16 acc0 = {0}, acc1 = {0};
#pragma unroll
            for (int kk = 0; kk < KS; ++kk) {
                const bf16x8 qf = St::frag(cur, 32 * par, kk, lane);
                acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ak[0][kk], qf, acc0, 0, 0, 0);
                if (need1) acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ak[1][kk], qf, acc1, 0, 0, 0);
            }
            const float l2 = s_lse[buf][32 * par + (lane & 31)];
            const int m = mt + (lane & 31);
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                if (a == 1 && !need1) continue;
                const f32x16 acc = a == 0 ? acc0 : acc1;
                const int klo = nk0 + 32 * a;
                if (mt >= klo + 31) {                      // every query of the half sees every key of the tile
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
        st.store(s_raw + (buf ^ 1) * St::BYTES);
        if (threadIdx.x < kStage) s_lse[buf ^ 1][threadIdx.x] = lreg;
        __syncthreads();
    }
    // sum the 32 query lanes and the two parities of every key through LDS, in a fixed order
    float* red = (float*)s_raw;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            red[((g * 2 + par) * 64 + 32 * a + acc_row(r, lane)) * 33 + (lane & 31)] = col[a][r];
    __syncthreads();
    if (threadIdx.x < kTile) {
        const int gg = threadIdx.x >> 6, kk = threadIdx.x & 63;
        float sum = 0.f;
#pragma unroll
        for (int pp = 0; pp < 2; ++pp)
#pragma unroll
            for (int j = 0; j < 32; ++j) sum += red[((gg * 2 + pp) * 64 + kk) * 33 + j];
        const int n = n0 + threadIdx.x;
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
