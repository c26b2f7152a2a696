// Causal prefill attention that also emits the log-sum-exp of every row (Sec. 3.1: the prefill phase
// attends over the whole prompt; Sec. 3.2 builds the importance from the same score matrix).  With the
// row lse handed over, the importance stage needs one pass over Q K^T instead of two.
//
//  prefill_attn_kernel  one workgroup = 128 queries of one (sequence, layer, head); a wavefront owns two
//                       tiles of 16 queries.  Keys and values stream through LDS 64 rows at a time
//                       (asynchronous global-to-LDS copies, double-buffered).  Both
//                       products run on the matrix cores with v_mfma_f32_16x16x32_bf16:
//                         S^T[16 keys x 16 queries] = K[16 x D] . Q^T            (A = K rows from LDS)
//                         O^T[16 d    x 16 queries] += V^T[16 d x 32 keys] . P^T (B = the probabilities,
//                                                       straight from the accumulators of S^T)
//                       In the accumulator layout a lane holds one query and 4 keys, so the softmax state
//                       is per lane and P^T needs no data movement: the 8 keys a lane contributes to a
//                       32-key product are its 4 keys of two consecutive S^T tiles.  V^T in that same key
//                       order comes from LDS with gfx950's transposing 64-bit read: 16 lanes point at
//                       4 keys x 16 columns of row-major V and each receives 4 keys of one column.
#include "pkv_common.hpp"

namespace pkv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef short v4i16_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) v4i16_t lds_v4i16_t;

struct PrefillParams {
    int B, L, H, Hkv, N, D;
    const bf16_t* q; Strides qs;
    const bf16_t* k; Strides ks;
    const bf16_t* v; Strides vs;
    const float* scale;   // [L]
    bf16_t* out;          // [B,L,H,N,D]
    float* lse;           // [B,L,H,N] natural log
};

constexpr int kPfQueries = 128;   // queries per workgroup (4 wavefronts x 2 tiles x 16)
constexpr int kPfKeys = 32;       // keys per product V^T . P^T (two S^T tiles)
constexpr int kPfStage = 64;      // keys per LDS stage

// two floats to packed bf16, round to nearest even (the hardware conversion of gfx950)
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    const f32x2_t f = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));
}

// 4 keys of one column of row-major V: lane r of a 16-lane group points at 4 consecutive columns of key
// r/4 (columns 4*(r%4) ...); lane i receives column i of keys 0..3.
__device__ __forceinline__ v4i16_t lds_read_tr(const unsigned char* p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16_t*)p);
}

template <int D>
__global__ void __launch_bounds__(256, 2)   // two wavefronts per SIMD: at most 256 registers, accumulators included
prefill_attn_kernel(PrefillParams p) {
    constexpr int ROWB = D * 2;
    constexpr int CPR = D / 8;            // 16-byte chunks per row
    constexpr int NJ = D / 32;            // MFMAs per S^T tile
    constexpr int NDT = D / 16;           // 16-column tiles of the output
    constexpr float kLog2e = 1.4426950408889634f, kLn2 = 0.6931471805599453f;
    // rows are stored unpadded; the 16-byte chunks of row r sit at chunk position c ^ (r & (CPR-1)), which
    // spreads both the fragment reads (16 rows x one chunk) and the transposing reads over all banks
    // two statically separate buffer pairs: while one is read, the asynchronous copy of the next stage
    // fills the other, and the compiler can see that the two do not alias
    __shared__ __attribute__((aligned(1024))) unsigned char sKa[kPfStage * ROWB];
    __shared__ __attribute__((aligned(1024))) unsigned char sVa[kPfStage * ROWB];
    __shared__ __attribute__((aligned(1024))) unsigned char sKb[kPfStage * ROWB];
    __shared__ __attribute__((aligned(1024))) unsigned char sVb[kPfStage * ROWB];

    const int heads = p.B * p.L * p.H;
    const int nqb = (p.N + kPfQueries - 1) / kPfQueries;
    const int qb = nqb - 1 - (int)(blockIdx.x / heads);    // the long (late) query blocks start first
    const int hh = blockIdx.x % heads;
    const int h = hh % p.H, l = (hh / p.H) % p.L, b = hh / (p.H * p.L);
    const int kvh = h / (p.H / p.Hkv);
    const bf16_t* qbase = p.q + p.qs.b * b + p.qs.l * l + p.qs.h * h;
    const bf16_t* kbase = p.k + p.ks.b * b + p.ks.l * l + p.ks.h * kvh;
    const bf16_t* vbase = p.v + p.vs.b * b + p.vs.l * l + p.vs.h * kvh;
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave;
    const int ln = lane & 15, kg = lane >> 4;
    const int q0 = qb * kPfQueries + wv * 32;               // first query of this wavefront
    const float qs = p.scale[l] * kLog2e;

    // the queries: B operand of the score products, [tile][d-slice]
    bf16x8_t qf[2][NJ];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        int row = q0 + 16 * t + ln;
        row = row < p.N ? row : p.N - 1;
#pragma unroll
        for (int j = 0; j < NJ; ++j)
            qf[t][j] = __builtin_bit_cast(bf16x8_t, *(const uint4*)(qbase + p.qs.n * row + 32 * j + 8 * kg));
    }
    f32x4_t o[2][NDT];
    float m_run[2], l_run[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        m_run[t] = -INFINITY; l_run[t] = 0.f;
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt) o[t][dt] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
    }

    const int last_q = min(p.N, (qb + 1) * kPfQueries) - 1;  // last query of the workgroup
    const int nst = last_q / kPfStage + 1;                   // stages that hold a key <= last_q

    // asynchronous copy of one stage (keys and values) into a buffer pair: gfx950's 16-byte global-to-LDS
    // load writes lane i's bytes to LDS[base + 16*i], so one instruction fills 1 KB of consecutive LDS and
    // the swizzle is applied on the global side
    constexpr int kInst = kPfStage * ROWB / 1024 / 4;        // copy instructions per wavefront and tensor
    auto issue = [&](int st, unsigned char* dK, unsigned char* dV) {
#pragma unroll
        for (int i = 0; i < kInst; ++i) {
            const int inst = wv * kInst + i;
            const int idx = inst * 64 + lane;
            const int r = idx / CPR, pos = idx % CPR;
            const int c = pos ^ (r & (CPR - 1));
            int row = st * kPfStage + r;
            row = row < p.N ? row : p.N - 1;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(kbase + p.ks.n * row + 8 * c),
                                             (__attribute__((address_space(3))) void*)(dK + inst * 1024), 16, 0, 0);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(vbase + p.vs.n * row + 8 * c),
                                             (__attribute__((address_space(3))) void*)(dV + inst * 1024), 16, 0, 0);
        }
    };

    auto step = [&](int st, const unsigned char* stK, const unsigned char* stV, unsigned char* nK, unsigned char* nV) {
        __builtin_amdgcn_s_waitcnt(0x0F70);                  // vmcnt(0): this wavefront's part of stage st has landed
        __syncthreads();                                     // ... and everybody's; the other pair is free again
        if (st + 1 < nst) issue(st + 1, nK, nV);
      for (int half = 0; half < kPfStage / kPfKeys; ++half) {
        const int key0 = st * kPfStage + half * kPfKeys;
        const unsigned char* sK = stK + half * kPfKeys * ROWB;
        const unsigned char* sV = stV + half * kPfKeys * ROWB;
        if (key0 > q0 + 31 || q0 >= p.N) return;             // every further key is in this wavefront's future
        const bool mask = key0 + kPfKeys - 1 > q0 || key0 + kPfKeys > p.N;

        // scores S^T = K . Q^T for the two key tiles of the stage and both query tiles
        f32x4_t s[2][2];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
            bf16x8_t kf[NJ];
            const int r = kt * 16 + ln;
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                const int pos = (4 * j + kg) ^ (r & (CPR - 1));
                kf[j] = __builtin_bit_cast(bf16x8_t, *(const uint4*)(sK + r * ROWB + pos * 16));
            }
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                s[t][kt] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int j = 0; j < NJ; ++j)
                    s[t][kt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[j], qf[t][j], s[t][kt], 0, 0, 0);
            }
        }
        // online softmax per query (= per lane column), probabilities as the B operand of the second product
        bf16x8_t pf[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int query = q0 + 16 * t + ln;
            float mx = -INFINITY;
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float sc = s[t][kt][r] * qs;
                    if (mask) {
                        const int key = key0 + 16 * kt + 4 * kg + r;
                        sc = (key <= query && key < p.N) ? sc : -INFINITY;
                    }
                    s[t][kt][r] = sc;
                    mx = fmaxf(mx, sc);
                }
            mx = fmaxf(mx, __shfl_xor(mx, 16, kWave));
            mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
            const float mnew = fmaxf(m_run[t], mx);
            // a query that has seen no key yet (only possible for padding queries beyond N) keeps its state
            const float corr = mnew == -INFINITY ? 1.f : __builtin_amdgcn_exp2f(m_run[t] - mnew);
            const float mref = mnew == -INFINITY ? 0.f : mnew;
            m_run[t] = mnew;
            float psum = 0.f;
            uint32_t pk[4];
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int r = 0; r < 4; r += 2) {
                    const float p0 = __builtin_amdgcn_exp2f(s[t][kt][r] - mref);
                    const float p1 = __builtin_amdgcn_exp2f(s[t][kt][r + 1] - mref);
                    psum += p0 + p1;
                    pk[kt * 2 + r / 2] = pack_bf16(p0, p1);
                }
            l_run[t] = l_run[t] * corr + psum;
            pf[t] = __builtin_bit_cast(bf16x8_t, make_uint4(pk[0], pk[1], pk[2], pk[3]));
            if (__builtin_amdgcn_ballot_w64(corr != 1.f)) {      // the running maximum moved for some query
#pragma unroll
                for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
                    for (int r = 0; r < 4; ++r) o[t][dt][r] *= corr;
            }
        }
        // O^T += V^T . P^T, one product per 16 output columns; the V^T operand serves both query tiles
        const int vr = 4 * kg + (ln >> 2);                   // key (within a 16-key tile) this lane points at
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt) {
            const int chunk = 2 * dt + ((ln & 3) >> 1), sub8 = (ln & 1) * 8;
            const v4i16_t a0 = lds_read_tr(sV + vr * ROWB + ((chunk ^ (vr & (CPR - 1))) * 16) + sub8);
            const v4i16_t a1 = lds_read_tr(sV + (16 + vr) * ROWB + ((chunk ^ ((16 + vr) & (CPR - 1))) * 16) + sub8);
            const bf16x8_t vf = __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(a0, a1, 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
            for (int t = 0; t < 2; ++t)
                o[t][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf[t], o[t][dt], 0, 0, 0);
        }
      }
    };

    issue(0, sKa, sVa);
    for (int st = 0; st < nst; st += 2) {
        step(st, sKa, sVa, sKb, sVb);
        if (st + 1 < nst) step(st + 1, sKb, sVb, sKa, sVa);
    }

    // epilogue: the four lane groups of a query hold partial row sums; the output tile is transposed
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        float lt = l_run[t];
        lt += __shfl_xor(lt, 16, kWave);
        lt += __shfl_xor(lt, 32, kWave);
        const int query = q0 + 16 * t + ln;
        if (query >= p.N) continue;
        const float inv = 1.f / lt;
        const size_t row = (size_t)hh * p.N + query;
        if (kg == 0) p.lse[row] = kLn2 * (m_run[t] + __builtin_amdgcn_logf(lt));
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt) {
            const uint32_t w0 = pack_bf16(o[t][dt][0] * inv, o[t][dt][1] * inv);
            const uint32_t w1 = pack_bf16(o[t][dt][2] * inv, o[t][dt][3] * inv);
            *(uint2*)(p.out + row * D + 16 * dt + 4 * kg) = make_uint2(w0, w1);
        }
    }
}

hipError_t launch_prefill_attn(const pkv_shape& s, const void* q, Strides qs, const void* k, Strides ks,
                               const void* v, Strides vs, const float* scale, void* out, float* lse,
                               hipStream_t st) {
    PrefillParams p;
    p.B = s.B; p.L = s.L; p.H = s.H; p.Hkv = s.Hkv; p.N = s.N; p.D = s.D;
    p.q = (const bf16_t*)q; p.qs = qs; p.k = (const bf16_t*)k; p.ks = ks; p.v = (const bf16_t*)v; p.vs = vs;
    p.scale = scale; p.out = (bf16_t*)out; p.lse = lse;
    const long long heads = (long long)s.B * s.L * s.H;
    const long long nqb = (s.N + kPfQueries - 1) / kPfQueries;
    const dim3 grid((unsigned)(heads * nqb));
    if (s.D == 128) hipLaunchKernelGGL(prefill_attn_kernel<128>, grid, dim3(256), 0, st, p);
    else hipLaunchKernelGGL(prefill_attn_kernel<64>, grid, dim3(256), 0, st, p);
    return hipGetLastError();
}

}  // namespace pkv
