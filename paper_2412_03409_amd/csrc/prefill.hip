// Causal prefill attention that also emits the log-sum-exp of every row (Sec. 3.1: the prefill phase
// attends over the whole prompt; Sec. 3.2 builds the importance from the same score matrix).  With the
// row lse handed over, the importance stage needs one pass over Q K^T instead of two.
//
//  prefill_attn_kernel  one workgroup = 128 queries of one (sequence, layer, head); a wavefront owns 32 of
//                       them.  Keys and values stream through LDS 64 rows at a time (asynchronous
//                       global-to-LDS copies, double-buffered).  Both products run on the matrix cores with
//                       v_mfma_f32_32x32x16_bf16:
//                         S^T[32 keys x 32 queries] = K[32 x D] . Q^T            (A = K rows from LDS)
//                         O^T[32 d    x 32 queries] += V^T[32 d x 16 keys] . P^T (B = the probabilities,
//                                                       straight from the accumulators of S^T)
//                       In the accumulator layout a lane holds one query and 16 keys, so the softmax state
//                       is per lane and P^T needs no data movement: the 8 keys a lane contributes to a
//                       16-key product are 8 consecutive accumulator registers.  V^T in that same key
//                       order comes from LDS with gfx950's transposing 64-bit read: 16 lanes point at
//                       4 keys x 16 columns of row-major V and each receives 4 keys of one column.
#include "pkv_common.hpp"

namespace pkv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
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

// Chunk swizzle of the staged rows: chunk c of row r sits at position c ^ swz(r).  The fragment reads of K
// touch 16 consecutive rows at one chunk, the transposing reads of V touch 4 consecutive rows at 4
// consecutive chunks; swapping the two low bit pairs of the row index sends both patterns to distinct banks.
template <int CPR>
__device__ __forceinline__ int swz(int r) {
    if constexpr (CPR == 16) return ((r & 3) << 2) | ((r >> 2) & 3);
    else return ((r & 1) << 2) | ((r >> 1) & 3);
}

template <int D>
__global__ void __launch_bounds__(256, 2)   // two wavefronts per SIMD: at most 256 registers, accumulators included
prefill_attn_kernel(PrefillParams p) {
    constexpr int ROWB = D * 2;
    constexpr int CPR = D / 8;            // 16-byte chunks per row
    constexpr int NJ = D / 16;            // MFMAs per S^T tile
    constexpr int NDT = D / 32;           // 32-column tiles of the output
    constexpr float kLog2e = 1.4426950408889634f, kLn2 = 0.6931471805599453f;
    // rows are stored unpadded, their 16-byte chunks swizzled (see swz).
    // Two statically separate buffer pairs: while one is read, the asynchronous copy of the next stage
    // fills the other, and the compiler can see that the two do not alias
    __shared__ __attribute__((aligned(1024))) unsigned char sKa[kPfStage * ROWB];
    __shared__ __attribute__((aligned(1024))) unsigned char sVa[kPfStage * ROWB];
    __shared__ __attribute__((aligned(1024))) unsigned char sKb[kPfStage * ROWB];
    __shared__ __attribute__((aligned(1024))) unsigned char sVb[kPfStage * ROWB];

    const int heads = p.B * p.L * p.H;
    const int nqb = (p.N + kPfQueries - 1) / kPfQueries;
    // The query blocks of one head run next to each other on one XCD (the hardware deals consecutive workgroups
    // out to the eight XCDs in turn) and share the head's K and V through that XCD's L2, as do the query heads
    // of one KV head; within a head the long (late) query blocks start first.
    const int per_xcd = (int)(gridDim.x / kXcds);         // a whole number of heads
    const int j = (int)(blockIdx.x % kXcds) * per_xcd + (int)(blockIdx.x / kXcds);
    const int qb = nqb - 1 - j % nqb;
    const int hh = j / nqb;
    if (hh >= heads) return;
    const int h = hh % p.H, l = (hh / p.H) % p.L, b = hh / (p.H * p.L);
    const int kvh = h / (p.H / p.Hkv);
    const bf16_t* qbase = p.q + p.qs.b * b + p.qs.l * l + p.qs.h * h;
    const bf16_t* kbase = p.k + p.ks.b * b + p.ks.l * l + p.ks.h * kvh;
    const bf16_t* vbase = p.v + p.vs.b * b + p.vs.l * l + p.vs.h * kvh;
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave;
    const int ln = lane & 31, hf = lane >> 5;               // MFMA operand row / column, and k-half
    const int q0 = qb * kPfQueries + wv * 32;               // first query of this wavefront
    const int query = q0 + ln;
    // a negative logit scale is moved into the queries (negation is exact in bf16), so that the running
    // maximum can be taken on the raw products
    const float sc_l = p.scale[l];
    const float qs = fabsf(sc_l) * kLog2e;
    const uint32_t sgn = sc_l < 0.f ? 0x80008000u : 0u;

    // the queries: B operand of the score products, one fragment per 16 columns of the head dimension
    bf16x8_t qf[NJ];
    {
        const int row = query < p.N ? query : p.N - 1;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            uint4 t = *(const uint4*)(qbase + p.qs.n * row + 16 * j + 8 * hf);
            t.x ^= sgn; t.y ^= sgn; t.z ^= sgn; t.w ^= sgn;
            qf[j] = __builtin_bit_cast(bf16x8_t, t);
        }
    }
    f32x16_t o[NDT];
    float m_run = -INFINITY, l_run = 0.f;
#pragma unroll
    for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;

    const int last_q = min(p.N, (qb + 1) * kPfQueries) - 1;  // last query of the workgroup
    const int nst = last_q / kPfStage + 1;                   // stages that hold a key <= last_q

    // asynchronous copy of one stage (keys and values) into a buffer pair: gfx950's 16-byte global-to-LDS
    // load writes lane i's bytes to LDS[base + 16*i], so one instruction fills 1 KB of consecutive LDS and
    // the swizzle is applied on the global side
    constexpr int kInst = kPfStage * ROWB / 1024 / 4;        // copy instructions per wavefront and tensor
    int cp_row[kInst], cp_col[kInst];                        // row within the stage and first element of the chunk
#pragma unroll
    for (int i = 0; i < kInst; ++i) {
        const int idx = (wv * kInst + i) * 64 + lane;
        const int r = idx / CPR, pos = idx % CPR;
        cp_row[i] = r;
        cp_col[i] = 8 * (pos ^ swz<CPR>(r));
    }
    const uint32_t ksn = (uint32_t)p.ks.n, vsn = (uint32_t)p.vs.n;   // N * stride < 2^31, checked by the launcher
    auto issue = [&](int st, unsigned char* dK, unsigned char* dV) {
#pragma unroll
        for (int i = 0; i < kInst; ++i) {
            int row = st * kPfStage + cp_row[i];
            row = row < p.N ? row : p.N - 1;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(kbase + ((uint32_t)row * ksn + (uint32_t)cp_col[i])),
                                             (__attribute__((address_space(3))) void*)(dK + (wv * kInst + i) * 1024), 16, 0, 0);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(vbase + ((uint32_t)row * vsn + (uint32_t)cp_col[i])),
                                             (__attribute__((address_space(3))) void*)(dV + (wv * kInst + i) * 1024), 16, 0, 0);
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

        // scores S^T[32 keys x 32 queries] = K . Q^T
        f32x16_t s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const int pos = (2 * j + hf) ^ swz<CPR>(ln);
            const bf16x8_t kf = __builtin_bit_cast(bf16x8_t, *(const uint4*)(sK + ln * ROWB + pos * 16));
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[j], s, 0, 0, 0);
        }
        // online softmax per query (= per lane column); register r holds key 8*(r/4) + 4*hf + r%4
        // (the running maximum m_run is kept in scaled units, log2 domain; the products stay raw)
        if (mask) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = key0 + 8 * (r >> 2) + 4 * hf + (r & 3);
                s[r] = (key <= query && key < p.N) ? s[r] : -INFINITY;
            }
        }
        float mx = s[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, kWave)) * qs;
        const float mnew = fmaxf(m_run, mx);
        // a query that has seen no key yet (only possible for padding queries beyond N) keeps its state
        const float corr = mnew == -INFINITY ? 1.f : __builtin_amdgcn_exp2f(m_run - mnew);
        const float mref = mnew == -INFINITY ? 0.f : mnew;
        m_run = mnew;
        // probabilities as the B operand of the second product: the 8 keys this lane contributes to the
        // 16-key product `sl` are registers 8*sl .. 8*sl+7, i.e. keys 16*sl + {4*hf .. 4*hf+3, 8+4*hf .. 8+4*hf+3}
        bf16x8_t pf[2];
        float psum = 0.f;
#pragma unroll
        for (int sl = 0; sl < 2; ++sl) {
            uint32_t pk[4];
#pragma unroll
            for (int e = 0; e < 8; e += 2) {
                const float p0 = __builtin_amdgcn_exp2f(fmaf(s[8 * sl + e], qs, -mref));
                const float p1 = __builtin_amdgcn_exp2f(fmaf(s[8 * sl + e + 1], qs, -mref));
                psum += p0 + p1;
                pk[e / 2] = pack_bf16(p0, p1);
            }
            pf[sl] = __builtin_bit_cast(bf16x8_t, make_uint4(pk[0], pk[1], pk[2], pk[3]));
        }
        l_run = l_run * corr + psum;
        if (__builtin_amdgcn_ballot_w64(corr != 1.f)) {      // the running maximum moved for some query
#pragma unroll
            for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[dt][r] *= corr;
        }
        // O^T[32 d x 32 queries] += V^T[32 d x 16 keys] . P^T.  The V^T operand in the key order above comes from
        // two transposing reads: the 16 lanes of a group point at 4 consecutive keys x 16 columns and each
        // receives the 4 keys of its own column
        const int g2 = (lane >> 4) & 1, i16 = lane & 15;
        const int vrow = 4 * hf + (i16 >> 2);                // key within the 16-key product this lane points at
        const int sub8 = (i16 & 1) * 8;
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt) {
            const int chunk = 4 * dt + 2 * g2 + ((i16 & 3) >> 1);
#pragma unroll
            for (int sl = 0; sl < 2; ++sl) {
                const int r0 = 16 * sl + vrow, r1 = r0 + 8;
                const v4i16_t a0 = lds_read_tr(sV + r0 * ROWB + ((chunk ^ swz<CPR>(r0)) * 16) + sub8);
                const v4i16_t a1 = lds_read_tr(sV + r1 * ROWB + ((chunk ^ swz<CPR>(r1)) * 16) + sub8);
                const bf16x8_t vf = __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(a0, a1, 0, 1, 2, 3, 4, 5, 6, 7));
                o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[sl], o[dt], 0, 0, 0);
            }
        }
      }
    };

    issue(0, sKa, sVa);
    for (int st = 0; st < nst; st += 2) {
        step(st, sKa, sVa, sKb, sVb);
        if (st + 1 < nst) step(st + 1, sKb, sVb, sKa, sVa);
    }

    // epilogue: the two halves of a query column hold partial row sums; the output tile is transposed:
    // register r of o[dt] is column 32*dt + 8*(r/4) + 4*hf + r%4 of this lane's query
    float lt = l_run;
    lt += __shfl_xor(lt, 32, kWave);
    if (query < p.N) {
        const float inv = 1.f / lt;
        const size_t row = (size_t)hh * p.N + query;
        if (hf == 0) p.lse[row] = kLn2 * (m_run + __builtin_amdgcn_logf(lt));
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const uint32_t w0 = pack_bf16(o[dt][4 * g] * inv, o[dt][4 * g + 1] * inv);
                const uint32_t w1 = pack_bf16(o[dt][4 * g + 2] * inv, o[dt][4 * g + 3] * inv);
                *(uint2*)(p.out + row * D + 32 * dt + 8 * g + 4 * hf) = make_uint2(w0, w1);
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
    const long long nblk = (heads + kXcds - 1) / kXcds * nqb * kXcds;   // whole heads per XCD
    if (nblk > 0x7fffffffll) return hipErrorInvalidValue;
    const dim3 grid((unsigned)nblk);
    if (s.D == 128) hipLaunchKernelGGL(prefill_attn_kernel<128>, grid, dim3(256), 0, st, p);
    else hipLaunchKernelGGL(prefill_attn_kernel<64>, grid, dim3(256), 0, st, p);
    return hipGetLastError();
}

}  // namespace pkv
