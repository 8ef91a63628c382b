// INT-FlashAttention forward (Algorithm 1) for gfx950: one fused kernel.
//
// Work split.  A workgroup of 4 wavefronts owns B_r = 128 query rows of one head, 32 per
// wavefront, and walks the key blocks of B_c = 128 keys in ascending order (Algorithm 1 lines
// 7-14).  K_j and V_j are staged once per workgroup in LDS; everything else lives in registers.
//
// Orientation.  Both GEMMs are computed transposed on v_mfma_i32_32x32x32_i8:
//     S^T = K_j Q_i^T   (A = K_j rows from LDS, B = Q_i rows held in registers)
//     O^T = V_j^T P^T   (A = V_j^T rows from LDS, B = P^T, the packed softmax block)
// The 32x32 accumulator gives lane (c, g) = (lane % 32, lane / 32) column c and rows
// 8*(v/4) + 4*g + v%4, v = 0..15.  With queries as columns, a lane owns ONE query and 16 keys per
// 32-key tile: row max and row sum are in-lane plus one exchange with lane ^ 32, and the 16 P
// bytes a lane produces for a 32-key tile are exactly the 16 contraction bytes the B operand
// of the second GEMM wants from that lane -- P never leaves registers.  The contraction index of
// O^T = V^T P^T may be permuted freely as long as both operands agree, so V_j^T is written to LDS
// with its keys in the order (tile, g, v) in which the accumulator layout delivers P.
//
// V_j is [keys, d] in HBM and the MFMA wants 16 consecutive KEYS per lane: the 4x4 byte transposes
// happen once per workgroup on the way into LDS (v_perm_b32), not per wavefront.
//
// Softmax in base 2: s_K is pre-multiplied by log2(e) when it is staged, the running max m2 is kept
// in log2 units and P = rint(exp2(a * s_Q - (m2 - log2 127))) with one v_exp_f32 per score.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <hip/hip_bf16.h>
#include <stdint.h>

#include "intfa.h"
#include "intfa_internal.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int BR = 128;       // query rows per workgroup
constexpr int BC = 128;       // keys per block: the B_c of Algorithm 1
constexpr int THREADS = 256;  // 4 wavefronts x 32 query rows
constexpr float LOG2E = 1.44269504088896340736f;
constexpr float LOG2_R = 6.98868468677216585326f;   // log2(127)
constexpr float RNE_MAGIC = 12582912.0f;            // 1.5 * 2^23: x + MAGIC rounds x to an integer (ties to even)

template <int D> struct Smem {
    alignas(16) int8_t k[BC * D];    // K_j, row = key, 16-byte chunks XOR-swizzled by row
    alignas(16) int8_t vt[D * BC];   // V_j^T, row = d, keys in accumulator order, chunks swizzled
    alignas(16) float sk[BC];        // s_K * log2(e) of the block
};

// 16-byte chunk c of K row `row` lives at chunk position k_swz(row, c): 8 consecutive rows hit 8
// different 16-byte slots of a 128-byte line, so a wavefront's 128-bit reads spread over all banks.
template <int D> __device__ __forceinline__ int k_swz(int row, int c) {
    return (D == 128) ? (c ^ (row & 7)) : (c ^ ((row >> 1) & 3));
}

// ---- staging: HBM -> LDS ------------------------------------------------------------------------
template <int D>
__device__ __forceinline__ void stage_k(const int8_t *__restrict__ Kh, int j0, int8_t *ks, int tid) {
    constexpr int CH = D / 16;
    constexpr int ITER = BC * CH / THREADS;
#pragma unroll
    for (int i = 0; i < ITER; ++i) {
        const int x = tid + THREADS * i;
        const int row = x / CH, c = x % CH;
        const v4i val = *reinterpret_cast<const v4i *>(Kh + static_cast<long>(j0 + row) * D + 16 * c);
        *reinterpret_cast<v4i *>(ks + row * D + k_swz<D>(row, c) * 16) = val;
    }
}

// A thread takes 4 consecutive keys x 16 d-bytes, transposes the four 4x4 byte blocks with v_perm
// and writes 16 dwords, each = 4 consecutive keys of one d column.  Key group kg = key / 4 goes to
// byte 32*(kg/8) + 16*(kg%2) + 4*((kg%8)/2) of the row: tile kg/8, half g = kg%2, dword (kg%8)/2,
// which is where accumulator row 8*(v/4) + 4*g + v%4 of that tile puts it.
template <int D>
__device__ __forceinline__ void stage_vt(const int8_t *__restrict__ Vh, int j0, int8_t *vt, int tid) {
    constexpr int CH = D / 16;
    if (tid < CH * 32) {
        const int dc = tid % CH, kg = tid / CH;
        v4i w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            w[i] = *reinterpret_cast<const v4i *>(Vh + static_cast<long>(j0 + 4 * kg + i) * D + 16 * dc);
        const int chunk = 2 * (kg >> 3) + (kg & 1);
        const int within = 4 * ((kg & 7) >> 1);
#pragma unroll
        for (int dw = 0; dw < 4; ++dw) {
            const uint32_t a0 = w[0][dw], a1 = w[1][dw], a2 = w[2][dw], a3 = w[3][dw];
            const uint32_t t0 = __builtin_amdgcn_perm(a1, a0, 0x05010400u);   // a0.b0 a1.b0 a0.b1 a1.b1
            const uint32_t t1 = __builtin_amdgcn_perm(a1, a0, 0x07030602u);   // a0.b2 a1.b2 a0.b3 a1.b3
            const uint32_t t2 = __builtin_amdgcn_perm(a3, a2, 0x05010400u);
            const uint32_t t3 = __builtin_amdgcn_perm(a3, a2, 0x07030602u);
            uint32_t o[4];
            o[0] = __builtin_amdgcn_perm(t2, t0, 0x05040100u);                // byte 0 of a0..a3
            o[1] = __builtin_amdgcn_perm(t2, t0, 0x07060302u);
            o[2] = __builtin_amdgcn_perm(t3, t1, 0x05040100u);
            o[3] = __builtin_amdgcn_perm(t3, t1, 0x07060302u);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int drow = 16 * dc + 4 * dw + c;
                *reinterpret_cast<uint32_t *>(vt + drow * BC + ((chunk ^ (drow & 7)) * 16) + within) = o[c];
            }
        }
    }
}

// ---- the two MFMA tile products -----------------------------------------------------------------
// S^T tile mt (keys 32*mt .. +31) x this wavefront's 32 queries, contraction over d.
template <int D>
__device__ __forceinline__ v16i gemm_kq_tile(const int8_t *ks, const v4i (&qf)[D / 32], int mt, int r, int g) {
    v16i acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    const int row = 32 * mt + r;
#pragma unroll
    for (int kk = 0; kk < D / 32; ++kk) {
        const v4i a = *reinterpret_cast<const v4i *>(ks + row * D + k_swz<D>(row, 2 * kk + g) * 16);
        acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, qf[kk], acc, 0, 0, 0);
    }
    return acc;
}

// O^T tile dt (d 32*dt .. +31) x 32 queries, contraction over the 128 keys of the block.
__device__ __forceinline__ v16i gemm_vp_tile(const int8_t *vt, const v4i (&pf)[BC / 32], int dt, int r, int g,
                                             v16i acc) {
    const int drow = 32 * dt + r;
#pragma unroll
    for (int mt = 0; mt < BC / 32; ++mt) {
        const v4i a = *reinterpret_cast<const v4i *>(vt + drow * BC + (((2 * mt + g) ^ (drow & 7)) * 16));
        acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, pf[mt], acc, 0, 0, 0);
    }
    return acc;
}

__device__ __forceinline__ float swap32(float x) {   // value held by lane ^ 32
    return __shfl_xor(x, 32);
}

// ---- output conversion --------------------------------------------------------------------------
template <typename T> struct Store4;
template <> struct Store4<float> {
    static __device__ __forceinline__ void put(float *p, float a, float b, float c, float d) {
        *reinterpret_cast<float4 *>(p) = make_float4(a, b, c, d);
    }
};
template <> struct Store4<__half> {
    static __device__ __forceinline__ void put(__half *p, float a, float b, float c, float d) {
        __half2 lo = __floats2half2_rn(a, b), hi = __floats2half2_rn(c, d);
        uint2 w;
        w.x = *reinterpret_cast<uint32_t *>(&lo);
        w.y = *reinterpret_cast<uint32_t *>(&hi);
        *reinterpret_cast<uint2 *>(p) = w;
    }
};
template <> struct Store4<__hip_bfloat16> {
    static __device__ __forceinline__ uint32_t rne(float x) {   // fp32 -> bf16 bits, round half to even
        uint32_t u = __float_as_uint(x);
        return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
    }
    static __device__ __forceinline__ void put(__hip_bfloat16 *p, float a, float b, float c, float d) {
        uint2 w;
        w.x = rne(a) | (rne(b) << 16);
        w.y = rne(c) | (rne(d) << 16);
        *reinterpret_cast<uint2 *>(p) = w;
    }
};

// ---- the fused kernel ---------------------------------------------------------------------------
template <int D, bool CAUSAL, typename OutT>
__global__ __launch_bounds__(THREADS) void int_flash_attn_fwd_kernel(
    const int8_t *__restrict__ Q, const int8_t *__restrict__ K, const int8_t *__restrict__ V,
    const float *__restrict__ sQ, const float *__restrict__ sK, const float *__restrict__ sV,
    int heads, int N, OutT *__restrict__ O) {
    __shared__ Smem<D> sm;
    constexpr int DT = D / 32;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r = lane & 31, g = lane >> 5;
    const int T_r = N / BR;

    // Workgroups go round-robin over the 8 XCDs by linear id; keep all query blocks of a head on
    // one XCD so its K/V stay in that XCD's L2.  Heavy (late) query blocks first under the mask.
    int head, qord;
    {
        const int L = blockIdx.x;
        if ((heads & 7) == 0) { const int s = L >> 3; head = (s / T_r) * 8 + (L & 7); qord = s % T_r; }
        else { head = L / T_r; qord = L % T_r; }
    }
    const int qb = CAUSAL ? (T_r - 1 - qord) : qord;
    const int q_local = 32 * wave + r;                           // this lane's query inside the block
    const long qrow = static_cast<long>(head) * N + qb * BR + q_local;

    const int8_t *Kh = K + static_cast<long>(head) * N * D;
    const int8_t *Vh = V + static_cast<long>(head) * N * D;
    const float *sKh = sK + static_cast<long>(head) * N;

    // line 5: Q_i and s_Q,i.  B operand: lane (r, g) holds bytes d = 32*kk + 16*g .. +15 of query r.
    v4i qf[D / 32];
#pragma unroll
    for (int kk = 0; kk < D / 32; ++kk)
        qf[kk] = *reinterpret_cast<const v4i *>(Q + qrow * D + 32 * kk + 16 * g);
    const float sq = sQ[qrow];

    // line 6
    float m2 = -INFINITY, l = 0.0f;
    float o[DT][16];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[dt][v] = 0.0f;

    const int nblocks = CAUSAL ? (qb + 1) : (N / BC);
    for (int jb = 0; jb < nblocks; ++jb) {                       // line 7
        const int j0 = jb * BC;
        __syncthreads();                                         // previous block fully consumed
        stage_k<D>(Kh, j0, sm.k, tid);                           // line 8
        stage_vt<D>(Vh, j0, sm.vt, tid);
        if (tid < BC) sm.sk[tid] = sKh[j0 + tid] * LOG2E;
        __syncthreads();

        // line 9: a = acc * s_K log2e (the positive per-row factor s_Q is applied after the max)
        float a[4][16];
        float bmax = -INFINITY;
        const bool diag = CAUSAL && (jb == qb);
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
            const v16i s = gemm_kq_tile<D>(sm.k, qf, mt, r, g);
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                const float4 skv = *reinterpret_cast<const float4 *>(&sm.sk[32 * mt + 8 * vq + 4 * g]);
                const float sk4[4] = {skv.x, skv.y, skv.z, skv.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float x = static_cast<float>(s[4 * vq + e]) * sk4[e];
                    if (diag && (32 * mt + 8 * vq + 4 * g + e > q_local)) x = -INFINITY;   // masked key
                    a[mt][4 * vq + e] = x;
                    bmax = fmaxf(bmax, x);
                }
            }
        }
        // line 10
        bmax = fmaxf(bmax, swap32(bmax));
        const float m_new = fmaxf(m2, bmax * sq);
        const float alpha = __builtin_amdgcn_exp2f(m2 - m_new);  // exp2(-inf) = 0 on the first block
        const float mm = m_new - LOG2_R;

        // line 11: P = rint(127 * 2^(a*s_Q - m_new)), packed 4 keys per dword in accumulator order
        v4i pf[4];
        uint32_t psum = 0;
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                uint32_t b[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(a[mt][4 * vq + e], sq, -mm));
                    b[e] = __float_as_uint(p + RNE_MAGIC);       // low byte = rint(p), 0..127
                }
                const uint32_t lo = __builtin_amdgcn_perm(b[1], b[0], 0x0c0c0400u);
                const uint32_t hi = __builtin_amdgcn_perm(b[3], b[2], 0x04000c0cu);
                const uint32_t w = lo | hi;
                psum = __builtin_amdgcn_sad_u8(w, 0u, psum);
                pf[mt][vq] = static_cast<int>(w);
            }
        }
        l = __builtin_fmaf(l, alpha, static_cast<float>(psum));                // line 12 (this lane's half of the keys)

        // line 13
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            const v16i zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
            const v16i pv = gemm_vp_tile(sm.vt, pf, dt, r, g, zero);
#pragma unroll
            for (int v = 0; v < 16; ++v) o[dt][v] = __builtin_fmaf(o[dt][v], alpha, static_cast<float>(pv[v]));
        }
        m2 = m_new;
    }

    // lines 15-17: O_i = diag(l)^-1 O s_V.  Lane (r, g) holds d = 32*dt + 8*(v/4) + 4*g + v%4.
    l += swap32(l);
    const float f = sV[head] / l;
    OutT *orow = O + qrow * D;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq)
            Store4<OutT>::put(orow + 32 * dt + 8 * vq + 4 * g, o[dt][4 * vq] * f, o[dt][4 * vq + 1] * f,
                              o[dt][4 * vq + 2] * f, o[dt][4 * vq + 3] * f);
}

// ---- test hooks: the same tile code, accumulators written out -------------------------------------
template <int D>
__global__ __launch_bounds__(THREADS) void debug_qk_kernel(const int8_t *__restrict__ Q, const int8_t *__restrict__ K,
                                                           int N, int *__restrict__ S) {
    __shared__ Smem<D> sm;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r = lane & 31, g = lane >> 5;
    const long qrow = blockIdx.x * BR + 32 * wave + r;
    const int j0 = blockIdx.y * BC;
    v4i qf[D / 32];
#pragma unroll
    for (int kk = 0; kk < D / 32; ++kk)
        qf[kk] = *reinterpret_cast<const v4i *>(Q + qrow * D + 32 * kk + 16 * g);
    stage_k<D>(K, j0, sm.k, tid);
    __syncthreads();
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
        const v16i s = gemm_kq_tile<D>(sm.k, qf, mt, r, g);
#pragma unroll
        for (int v = 0; v < 16; ++v)
            S[qrow * N + j0 + 32 * mt + 8 * (v >> 2) + 4 * g + (v & 3)] = s[v];
    }
}

template <int D>
__global__ __launch_bounds__(THREADS) void debug_pv_kernel(const int8_t *__restrict__ P, const int8_t *__restrict__ V,
                                                           int N, int *__restrict__ PV) {
    __shared__ Smem<D> sm;
    constexpr int DT = D / 32;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r = lane & 31, g = lane >> 5;
    const long qrow = blockIdx.x * BR + 32 * wave + r;
    v16i acc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) acc[dt] = v16i{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    for (int j0 = 0; j0 < N; j0 += BC) {
        __syncthreads();
        stage_vt<D>(V, j0, sm.vt, tid);
        __syncthreads();
        v4i pf[4];                                   // the layout the fused kernel builds in registers
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int vq = 0; vq < 4; ++vq)
                pf[mt][vq] = *reinterpret_cast<const int *>(P + qrow * N + j0 + 32 * mt + 8 * vq + 4 * g);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) acc[dt] = gemm_vp_tile(sm.vt, pf, dt, r, g, acc[dt]);
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) PV[qrow * D + 32 * dt + 8 * (v >> 2) + 4 * g + (v & 3)] = acc[dt][v];
}

// ---- host side ----------------------------------------------------------------------------------
hipStream_t g_stream = nullptr;

template <int D, bool CAUSAL, typename OutT>
int launch_fwd(const int8_t *Q, const int8_t *K, const int8_t *V, const float *sQ, const float *sK, const float *sV,
               int heads, int N, void *O, hipStream_t st) {
    const long wgs = static_cast<long>(heads) * (N / BR);
    hipLaunchKernelGGL((int_flash_attn_fwd_kernel<D, CAUSAL, OutT>), dim3(static_cast<unsigned>(wgs)), dim3(THREADS), 0,
                       st, Q, K, V, sQ, sK, sV, heads, N, static_cast<OutT *>(O));
    return hipGetLastError() == hipSuccess ? IFA_OK : IFA_ERR_HIP;
}

template <int D, bool CAUSAL>
int launch_fwd_dtype(const int8_t *Q, const int8_t *K, const int8_t *V, const float *sQ, const float *sK,
                     const float *sV, int heads, int N, void *O, int o_dtype, hipStream_t st) {
    switch (o_dtype) {
    case IFA_F32: return launch_fwd<D, CAUSAL, float>(Q, K, V, sQ, sK, sV, heads, N, O, st);
    case IFA_F16: return launch_fwd<D, CAUSAL, __half>(Q, K, V, sQ, sK, sV, heads, N, O, st);
    default: return launch_fwd<D, CAUSAL, __hip_bfloat16>(Q, K, V, sQ, sK, sV, heads, N, O, st);
    }
}

}  // namespace

hipStream_t ifa_current_stream() { return g_stream; }

extern "C" const char *ifa_status_str(int status) {
    switch (status) {
    case IFA_OK: return "IFA_OK";
    case IFA_ERR_NULL: return "IFA_ERR_NULL: null pointer argument";
    case IFA_ERR_SHAPE: return "IFA_ERR_SHAPE: non-positive or overflowing size";
    case IFA_ERR_DTYPE: return "IFA_ERR_DTYPE: unknown dtype";
    case IFA_ERR_UNSUPPORTED: return "IFA_ERR_UNSUPPORTED: shape, granularity or alignment not supported";
    case IFA_ERR_HIP: return "IFA_ERR_HIP: HIP launch failed";
    default: return "unknown ifa_status";
    }
}

extern "C" int ifa_set_stream(void *hip_stream) {
    g_stream = static_cast<hipStream_t>(hip_stream);
    return IFA_OK;
}

extern "C" int ifa_block_cols(int d, int causal) {
    (void)causal;
    return (d == 64 || d == 128) ? BC : 0;
}

extern "C" int int_flash_attn_fwd_ex(const signed char *Q_i8, const signed char *K_i8, const signed char *V_i8,
                                     const float *s_Q, const float *s_K, const float *s_V, int B, int H, int N, int d,
                                     int causal, void *O, int o_dtype, void *hip_stream) {
    if (!Q_i8 || !K_i8 || !V_i8 || !s_Q || !s_K || !s_V || !O) return IFA_ERR_NULL;
    if (B <= 0 || H <= 0 || N <= 0 || d <= 0) return IFA_ERR_SHAPE;
    const long heads = static_cast<long>(B) * H;
    if (heads > (1L << 40) / N / d) return IFA_ERR_SHAPE;
    if (o_dtype < IFA_F32 || o_dtype > IFA_BF16) return IFA_ERR_DTYPE;
    if ((d != 64 && d != 128) || N % BR != 0 || N % BC != 0) return IFA_ERR_UNSUPPORTED;
    if (heads * (N / BR) > 0x7fffffffL) return IFA_ERR_UNSUPPORTED;
    if (!ifa_aligned16(Q_i8) || !ifa_aligned16(K_i8) || !ifa_aligned16(V_i8) || !ifa_aligned16(O) ||
        (reinterpret_cast<uintptr_t>(s_Q) & 3) || (reinterpret_cast<uintptr_t>(s_K) & 3) ||
        (reinterpret_cast<uintptr_t>(s_V) & 3))
        return IFA_ERR_UNSUPPORTED;
    const int8_t *Q = reinterpret_cast<const int8_t *>(Q_i8);
    const int8_t *K = reinterpret_cast<const int8_t *>(K_i8);
    const int8_t *V = reinterpret_cast<const int8_t *>(V_i8);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const int hd = static_cast<int>(heads);
    if (d == 128)
        return causal ? launch_fwd_dtype<128, true>(Q, K, V, s_Q, s_K, s_V, hd, N, O, o_dtype, st)
                      : launch_fwd_dtype<128, false>(Q, K, V, s_Q, s_K, s_V, hd, N, O, o_dtype, st);
    return causal ? launch_fwd_dtype<64, true>(Q, K, V, s_Q, s_K, s_V, hd, N, O, o_dtype, st)
                  : launch_fwd_dtype<64, false>(Q, K, V, s_Q, s_K, s_V, hd, N, O, o_dtype, st);
}

extern "C" int int_flash_attn_fwd(const signed char *Q_i8, const signed char *K_i8, const signed char *V_i8,
                                  const float *s_Q, const float *s_K, const float *s_V, int B, int H, int N, int d,
                                  int causal, void *O) {
    return int_flash_attn_fwd_ex(Q_i8, K_i8, V_i8, s_Q, s_K, s_V, B, H, N, d, causal, O, IFA_F16, g_stream);
}

extern "C" int ifa_debug_qk_i32(const signed char *Q_i8, const signed char *K_i8, int N, int d, int *S_i32) {
    if (!Q_i8 || !K_i8 || !S_i32) return IFA_ERR_NULL;
    if (N <= 0 || d <= 0) return IFA_ERR_SHAPE;
    if ((d != 64 && d != 128) || N % BR != 0 || N > 32768) return IFA_ERR_UNSUPPORTED;
    if (!ifa_aligned16(Q_i8) || !ifa_aligned16(K_i8) || (reinterpret_cast<uintptr_t>(S_i32) & 3)) return IFA_ERR_UNSUPPORTED;
    const int8_t *Q = reinterpret_cast<const int8_t *>(Q_i8);
    const int8_t *K = reinterpret_cast<const int8_t *>(K_i8);
    const dim3 grid(N / BR, N / BC);
    if (d == 128) hipLaunchKernelGGL(debug_qk_kernel<128>, grid, dim3(THREADS), 0, g_stream, Q, K, N, S_i32);
    else hipLaunchKernelGGL(debug_qk_kernel<64>, grid, dim3(THREADS), 0, g_stream, Q, K, N, S_i32);
    return hipGetLastError() == hipSuccess ? IFA_OK : IFA_ERR_HIP;
}

extern "C" int ifa_debug_pv_i32(const signed char *P_i8, const signed char *V_i8, int N, int d, int *PV_i32) {
    if (!P_i8 || !V_i8 || !PV_i32) return IFA_ERR_NULL;
    if (N <= 0 || d <= 0) return IFA_ERR_SHAPE;
    if ((d != 64 && d != 128) || N % BR != 0 || N > 32768) return IFA_ERR_UNSUPPORTED;
    if (!ifa_aligned16(P_i8) || !ifa_aligned16(V_i8) || (reinterpret_cast<uintptr_t>(PV_i32) & 3)) return IFA_ERR_UNSUPPORTED;
    const int8_t *P = reinterpret_cast<const int8_t *>(P_i8);
    const int8_t *V = reinterpret_cast<const int8_t *>(V_i8);
    const dim3 grid(N / BR);
    if (d == 128) hipLaunchKernelGGL(debug_pv_kernel<128>, grid, dim3(THREADS), 0, g_stream, P, V, N, PV_i32);
    else hipLaunchKernelGGL(debug_pv_kernel<64>, grid, dim3(THREADS), 0, g_stream, P, V, N, PV_i32);
    return hipGetLastError() == hipSuccess ? IFA_OK : IFA_ERR_HIP;
}
