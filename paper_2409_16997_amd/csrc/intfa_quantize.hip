// Symmetric INT8 quantizers of Section 3.2 (S = absmax / R, R = 127), gfx950.
//
// Both are HBM-streaming kernels: every element is read once (twice for V, whose scale needs
// the whole head first) and written once as a byte.  A lane owns 8 consecutive elements, so
// loads are 128-bit for fp16/bf16 and 2 x 128-bit for fp32, stores are 64-bit, and a row of
// d elements is d/8 adjacent lanes whose absmax is combined with DPP lane shuffles.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <hip/hip_bf16.h>
#include <stdint.h>

#include "intfa.h"
#include "intfa_internal.h"

namespace {

// ---- 8 consecutive elements of any supported dtype, widened exactly to fp32 ------------------
template <typename T> struct Load8;

template <> struct Load8<float> {
    static __device__ __forceinline__ void get(const void *p, long idx, float (&x)[8]) {
        const float4 *q = reinterpret_cast<const float4 *>(static_cast<const float *>(p) + idx);
        float4 a = q[0], b = q[1];
        x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
    }
};
template <> struct Load8<__half> {
    static __device__ __forceinline__ void get(const void *p, long idx, float (&x)[8]) {
        uint4 raw = *reinterpret_cast<const uint4 *>(static_cast<const __half *>(p) + idx);
        const __half2 *h = reinterpret_cast<const __half2 *>(&raw);
#pragma unroll
        for (int i = 0; i < 4; ++i) { float2 f = __half22float2(h[i]); x[2 * i] = f.x; x[2 * i + 1] = f.y; }
    }
};
template <> struct Load8<__hip_bfloat16> {
    static __device__ __forceinline__ void get(const void *p, long idx, float (&x)[8]) {
        uint4 raw = *reinterpret_cast<const uint4 *>(static_cast<const __hip_bfloat16 *>(p) + idx);
        const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {                 // bf16 -> fp32 is a 16-bit shift
            x[2 * i] = __uint_as_float(w[i] << 16);
            x[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
};

__device__ __forceinline__ float absmax8(const float (&x)[8]) {
    float a = fmaxf(fabsf(x[0]), fabsf(x[1]));
#pragma unroll
    for (int i = 2; i < 8; ++i) a = fmaxf(a, fabsf(x[i]));
    return a;
}

// q = clamp(rint(x * inv), -127, 127) for 8 values, packed little-endian into two dwords.
__device__ __forceinline__ uint2 quant8(const float (&x)[8], float inv) {
    uint32_t w[2] = {0u, 0u};
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        float t = rintf(x[i] * inv);
        t = fminf(fmaxf(t, -127.0f), 127.0f);
        w[i >> 2] |= (static_cast<uint32_t>(static_cast<int>(t)) & 0xffu) << (8 * (i & 3));
    }
    return make_uint2(w[0], w[1]);
}

// max over the aligned group of `LPR` adjacent lanes (LPR a power of two <= 64), result in all.
template <int LPR>
__device__ __forceinline__ float group_max(float a) {
    // quad_perm [1,0,3,2] and [2,3,0,1], then mirrors inside 8 and 16 lanes: DPP, no LDS.
    if (LPR >= 2) a = fmaxf(a, __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(a), 0xB1, 0xf, 0xf, true)));
    if (LPR >= 4) a = fmaxf(a, __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(a), 0x4E, 0xf, 0xf, true)));
    if (LPR >= 8) a = fmaxf(a, __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(a), 0x141, 0xf, 0xf, true)));  // row_half_mirror
    if (LPR >= 16) a = fmaxf(a, __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(a), 0x140, 0xf, 0xf, true))); // row_mirror
    if (LPR >= 32) a = fmaxf(a, __shfl_xor(a, 16));
    if (LPR >= 64) a = fmaxf(a, __shfl_xor(a, 32));
    return a;
}

// value held by lane ^ M (M a power of two < 64): DPP inside a quad, the LDS crossbar (no memory access) beyond
template <int M> __device__ __forceinline__ float lane_xor(float x) {
    const int v = __float_as_int(x);
    if (M == 1) return __int_as_float(__builtin_amdgcn_mov_dpp(v, 0xB1, 0xf, 0xf, true));        // quad_perm [1,0,3,2]
    if (M == 2) return __int_as_float(__builtin_amdgcn_mov_dpp(v, 0x4E, 0xf, 0xf, true));        // quad_perm [2,3,0,1]
    if (M == 4) return __int_as_float(__builtin_amdgcn_ds_swizzle(v, 0x101F));                   // bit mode: xor 4
    if (M == 8) return __int_as_float(__builtin_amdgcn_ds_swizzle(v, 0x201F));
    if (M == 16) return __int_as_float(__builtin_amdgcn_ds_swizzle(v, 0x401F));
    return __shfl_xor(x, 32);
}

// One butterfly stage of the Walsh-Hadamard transform across lanes: elements 8*sub + i and 8*(sub ^ M) + i.
// The lane with bit M clear holds a and keeps a + b, the other holds b and keeps a - b.
template <int M, int LPR> __device__ __forceinline__ void hadamard_lane_stage(float (&x)[8], int sub) {
    if (M < LPR) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float p = lane_xor<M>(x[i]);
            x[i] = (sub & M) ? (p - x[i]) : (x[i] + p);
        }
    }
}

// Unnormalized Walsh-Hadamard transform (Sylvester order) of a row of 8*LPR elements spread over LPR lanes,
// stages h = 1, 2, 4 inside the lane's 8 registers, then h = 8, 16, ... across lanes, all in fp32.
template <int LPR> __device__ __forceinline__ void hadamard_row(float (&x)[8], int sub) {
#pragma unroll
    for (int h = 1; h < 8; h <<= 1)
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if ((i & h) == 0) {
                const float a = x[i], b = x[i + h];
                x[i] = a + b;
                x[i + h] = a - b;
            }
    hadamard_lane_stage<1, LPR>(x, sub);
    hadamard_lane_stage<2, LPR>(x, sub);
    hadamard_lane_stage<4, LPR>(x, sub);
    hadamard_lane_stage<8, LPR>(x, sub);
    hadamard_lane_stage<16, LPR>(x, sub);
    hadamard_lane_stage<32, LPR>(x, sub);
}

// ---- token-level: one row = LPR lanes ---------------------------------------------------------
// One launch serves up to two tensors of the same shape (Q and K of a step), can clear an array of words on the side
// (the absmax slots the tensor-level quantizer of V accumulates into afterwards) and can carry the first pass of that
// tensor-level quantizer along (HeadJob): blockIdx.y picks the job.
struct TokenJob {
    const void *X;
    int8_t *Xq;
    float *scale;
    float scale_mul;
};
// First pass of the tensor-level quantizer without atomics and without slots to clear: HEAD_PARTS workgroups per head
// each take a contiguous part of the head and leave the absmax of their part (fp32 bits) in the LAST 4 * HEAD_PARTS
// bytes of that head's OUTPUT codes, which nobody writes before head_tail_finalize_kernel does (it reads them first).
constexpr int HEAD_PARTS = 8;
struct HeadJob {
    const void *X;       // [heads, per_head]; null: no such job in this launch
    int8_t *Xq;
    long per_head;
    int heads;
};
template <typename T>
__device__ __forceinline__ void head_partial_absmax(const HeadJob &hj) {
    if (blockIdx.x >= static_cast<unsigned>(hj.heads) * HEAD_PARTS) return;
    const long head = blockIdx.x / HEAD_PARTS;
    const int part = blockIdx.x % HEAD_PARTS;
    const long chunks = hj.per_head / 8, per_part = (chunks + HEAD_PARTS - 1) / HEAD_PARTS;
    const long c0 = part * per_part, c1 = (c0 + per_part < chunks) ? c0 + per_part : chunks;
    float a = 0.0f;
#pragma unroll 8
    for (long c = c0 + threadIdx.x; c < c1; c += 256) {
        float x[8];
        Load8<T>::get(hj.X, head * hj.per_head + 8 * c, x);
        a = fmaxf(a, absmax8(x));
    }
    a = group_max<64>(a);
    __shared__ float wmax[4];
    if ((threadIdx.x & 63) == 0) wmax[threadIdx.x >> 6] = a;
    __syncthreads();
    if (threadIdx.x == 0)
        reinterpret_cast<unsigned *>(hj.Xq + (head + 1) * hj.per_head - 4 * HEAD_PARTS)[part] =
            __float_as_uint(fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3])));
}

template <typename T, int LPR, bool HADAMARD>
__global__ __launch_bounds__(256) void quantize_tokenwise_kernel(TokenJob j0, TokenJob j1, long rows,
                                                                 unsigned *__restrict__ clear, long clear_words, HeadJob hj) {
    constexpr int D = LPR * 8;
    constexpr int ROWS_PER_BLOCK = 256 / LPR;
    // the head job, if any, comes last in dispatch order: V is then the most recently read tensor when the second pass
    // of its quantizer starts, and that pass finds most of it in the Infinity Cache
    const int y = static_cast<int>(blockIdx.y);
    if (hj.X && y == static_cast<int>(gridDim.y) - 1) {
        head_partial_absmax<T>(hj);
        return;
    }
    const TokenJob job = y == 0 ? j0 : j1;
    const int sub = threadIdx.x % LPR;
    if (y == 0)
        for (long i = static_cast<long>(blockIdx.x) * 256 + threadIdx.x; i < clear_words; i += static_cast<long>(gridDim.x) * 256)
            clear[i] = 0u;
    const long row_stride = static_cast<long>(gridDim.x) * ROWS_PER_BLOCK;
    for (long row = static_cast<long>(blockIdx.x) * ROWS_PER_BLOCK + threadIdx.x / LPR; row < rows;
         row += row_stride) {
        float x[8];
        const long idx = row * D + sub * 8;
        Load8<T>::get(job.X, idx, x);
        if (HADAMARD) hadamard_row<LPR>(x, sub);
        const float a = group_max<LPR>(absmax8(x));
        const float inv = (a == 0.0f) ? 0.0f : 127.0f / a;
        *reinterpret_cast<uint2 *>(job.Xq + idx) = quant8(x, inv);
        if (sub == 0) job.scale[row] = ((a == 0.0f) ? 1.0f : a / 127.0f) * job.scale_mul;
    }
}

// ---- tensor-level: absmax of a head, then quantize ---------------------------------------------
// |x| >= 0, so the fp32 bit pattern orders like the value and an integer atomic max works.
template <typename T>
__global__ __launch_bounds__(256) void head_absmax_kernel(const void *__restrict__ X, long per_head,
                                                          unsigned *__restrict__ amax_bits, int global_scale) {
    const long head = blockIdx.y;
    const long base = head * per_head;
    float a = 0.0f;
    for (long i = (static_cast<long>(blockIdx.x) * 256 + threadIdx.x) * 8; i < per_head;
         i += static_cast<long>(gridDim.x) * 256 * 8) {
        float x[8];
        Load8<T>::get(X, base + i, x);
        a = fmaxf(a, absmax8(x));
    }
    a = group_max<64>(a);
    __shared__ float wmax[4];
    if ((threadIdx.x & 63) == 0) wmax[threadIdx.x >> 6] = a;
    __syncthreads();
    if (threadIdx.x == 0) {
        a = fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3]));
        // Atomics on one address serialise (hundreds of workgroups per head): look first.  The slot only grows, so a
        // value read here, however stale, is a lower bound of the final one and skipping below it loses nothing.
        unsigned *slot = amax_bits + (global_scale ? 0 : head);
        if (__float_as_uint(a) > __builtin_nontemporal_load(slot)) atomicMax(slot, __float_as_uint(a));
    }
}

template <typename T>
__global__ __launch_bounds__(256) void head_quantize_kernel(const void *__restrict__ X, long per_head,
                                                            const unsigned *__restrict__ amax_bits,
                                                            int8_t *__restrict__ Xq, int global_scale) {
    const long head = blockIdx.y;
    const long base = head * per_head;
    const float a = __uint_as_float(amax_bits[global_scale ? 0 : head]);
    const float inv = (a == 0.0f) ? 0.0f : 127.0f / a;
    for (long i = (static_cast<long>(blockIdx.x) * 256 + threadIdx.x) * 8; i < per_head;
         i += static_cast<long>(gridDim.x) * 256 * 8) {
        float x[8];
        Load8<T>::get(X, base + i, x);
        *reinterpret_cast<uint2 *>(Xq + base + i) = quant8(x, inv);
    }
}

// Second pass after head_partial_absmax: everything but the last 4 * HEAD_PARTS elements of the head (where the partial
// maxima still sit).
template <typename T>
__global__ __launch_bounds__(256) void head_quantize_from_parts_kernel(const void *__restrict__ X, long per_head, int8_t *__restrict__ Xq) {
    const long head = blockIdx.y;
    const long base = head * per_head;
    const unsigned *parts = reinterpret_cast<const unsigned *>(Xq + base + per_head - 4 * HEAD_PARTS);
    unsigned bits = 0u;
#pragma unroll
    for (int p = 0; p < HEAD_PARTS; ++p) bits = max(bits, parts[p]);   // |x| >= 0: the bit patterns order like the values
    const float a = __uint_as_float(bits);
    const float inv = (a == 0.0f) ? 0.0f : 127.0f / a;
    for (long i = (static_cast<long>(blockIdx.x) * 256 + threadIdx.x) * 8; i < per_head - 4 * HEAD_PARTS;
         i += static_cast<long>(gridDim.x) * 256 * 8) {
        float x[8];
        Load8<T>::get(X, base + i, x);
        *reinterpret_cast<uint2 *>(Xq + base + i) = quant8(x, inv);
    }
}

// Last pass: one thread per head reads the partial maxima, then writes the scale and the head's last 4 * HEAD_PARTS codes
// over them.
template <typename T>
__global__ __launch_bounds__(64) void head_tail_finalize_kernel(const void *__restrict__ X, long per_head, int8_t *__restrict__ Xq,
                                                                float *__restrict__ scale, long heads) {
    const long head = static_cast<long>(blockIdx.x) * 64 + threadIdx.x;
    if (head >= heads) return;
    const long tail = head * per_head + per_head - 4 * HEAD_PARTS;
    const unsigned *parts = reinterpret_cast<const unsigned *>(Xq + tail);
    unsigned bits = 0u;
#pragma unroll
    for (int p = 0; p < HEAD_PARTS; ++p) bits = max(bits, parts[p]);
    const float a = __uint_as_float(bits);
    const float inv = (a == 0.0f) ? 0.0f : 127.0f / a;
    uint2 q[4 * HEAD_PARTS / 8];
#pragma unroll
    for (int k = 0; k < 4 * HEAD_PARTS / 8; ++k) {
        float x[8];
        Load8<T>::get(X, tail + 8 * k, x);
        q[k] = quant8(x, inv);
    }
#pragma unroll
    for (int k = 0; k < 4 * HEAD_PARTS / 8; ++k) *reinterpret_cast<uint2 *>(Xq + tail + 8 * k) = q[k];
    scale[head] = (a == 0.0f) ? 1.0f : a / 127.0f;
}

// ---- block-level: one scale per (head, block of `block` keys), single pass -----------------------
// A workgroup owns one block: at most 128 keys x 128 channels = 16384 elements = 8 chunks of 8 per thread,
// held in registers between the absmax and the rounding, so the activations are read once.
template <typename T>
__global__ __launch_bounds__(256) void block_quantize_kernel(const void *__restrict__ X, long N, int d, int block,
                                                             int8_t *__restrict__ Xq, float *__restrict__ scale) {
    const long head = blockIdx.y, jb = blockIdx.x;
    const long first = head * N * d + jb * static_cast<long>(block) * d;     // first element of the block
    const long keys = (N - jb * block < block) ? (N - jb * block) : block;
    const int chunks = static_cast<int>(keys * d / 8);
    float x[8][8];
    float a = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int c = threadIdx.x + 256 * i;
        if (c < chunks) {
            Load8<T>::get(X, first + 8L * c, x[i]);
            a = fmaxf(a, absmax8(x[i]));
        }
    }
    a = group_max<64>(a);
    __shared__ float wmax[4];
    if ((threadIdx.x & 63) == 0) wmax[threadIdx.x >> 6] = a;
    __syncthreads();
    a = fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3]));
    const float inv = (a == 0.0f) ? 0.0f : 127.0f / a;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int c = threadIdx.x + 256 * i;
        if (c < chunks) *reinterpret_cast<uint2 *>(Xq + first + 8L * c) = quant8(x[i], inv);
    }
    if (threadIdx.x == 0) scale[head * gridDim.x + jb] = (a == 0.0f) ? 1.0f : a / 127.0f;
}

__global__ void zero_words_kernel(unsigned *p, long n) {
    const long i = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

// absmax bits -> scale, in place.  One block; slot 0 is read by every thread before any write.
__global__ void head_scale_finalize_kernel(float *scale, long heads, int global_scale) {
    const float a0 = __uint_as_float(reinterpret_cast<const unsigned *>(scale)[0]);
    __syncthreads();
    for (long h = threadIdx.x; h < heads; h += blockDim.x) {
        const float a = global_scale ? a0 : __uint_as_float(reinterpret_cast<const unsigned *>(scale)[h]);
        scale[h] = (a == 0.0f) ? 1.0f : a / 127.0f;
    }
}

template <typename T, bool HADAMARD>
int launch_tokenwise(const TokenJob &j0, const TokenJob &j1, int jobs, long rows, int d, unsigned *clear, long clear_words,
                     const HeadJob &hj, hipStream_t st) {
    const int lpr = d / 8;
    const long rows_per_block = 256 / lpr;
    long blocks = (rows + rows_per_block - 1) / rows_per_block;
    const long cap = 256L * 64 / jobs;                   // grid-stride beyond 64 blocks per CU (4 to 64 measured alike)
    if (blocks > cap) blocks = cap;
    if (hj.X && blocks < static_cast<long>(hj.heads) * HEAD_PARTS) blocks = static_cast<long>(hj.heads) * HEAD_PARTS;
    const dim3 grid(static_cast<unsigned>(blocks), static_cast<unsigned>(jobs + (hj.X ? 1 : 0))), block(256);
    switch (lpr) {
    case 4: hipLaunchKernelGGL((quantize_tokenwise_kernel<T, 4, HADAMARD>), grid, block, 0, st, j0, j1, rows, clear, clear_words, hj); break;
    case 8: hipLaunchKernelGGL((quantize_tokenwise_kernel<T, 8, HADAMARD>), grid, block, 0, st, j0, j1, rows, clear, clear_words, hj); break;
    case 16: hipLaunchKernelGGL((quantize_tokenwise_kernel<T, 16, HADAMARD>), grid, block, 0, st, j0, j1, rows, clear, clear_words, hj); break;
    case 32: hipLaunchKernelGGL((quantize_tokenwise_kernel<T, 32, HADAMARD>), grid, block, 0, st, j0, j1, rows, clear, clear_words, hj); break;
    case 64: hipLaunchKernelGGL((quantize_tokenwise_kernel<T, 64, HADAMARD>), grid, block, 0, st, j0, j1, rows, clear, clear_words, hj); break;
    default: return IFA_ERR_UNSUPPORTED;
    }
    return hipGetLastError() == hipSuccess ? IFA_OK : IFA_ERR_HIP;
}

template <typename T>
int launch_headwise(const void *X, long heads, long per_head, int8_t *Xq, float *scale, int global_scale,
                    hipStream_t st, bool slots_cleared = false) {
    unsigned *bits = reinterpret_cast<unsigned *>(scale);
    if (!slots_cleared)
        hipLaunchKernelGGL(zero_words_kernel, dim3(static_cast<unsigned>((heads + 255) / 256)), dim3(256), 0, st, bits, heads);
    long bx = (per_head / 8 + 255) / 256;
    // About 4 workgroups per CU in total: measured on MI355X (c3's V, 134 MB) the two passes take 92 us with 1 per
    // CU, 64 with 2, 57 with 4 or 8, 64 with 16, 72 with 32 -- more workgroups only add atomics on the head's slot.
    const long cap = (256L * 4 + heads - 1) / heads;
    if (bx > cap) bx = cap;
    if (bx < 1) bx = 1;
    const dim3 grid(static_cast<unsigned>(bx), static_cast<unsigned>(heads)), block(256);
    hipLaunchKernelGGL((head_absmax_kernel<T>), grid, block, 0, st, X, per_head, bits, global_scale);
    hipLaunchKernelGGL((head_quantize_kernel<T>), grid, block, 0, st, X, per_head, bits, Xq, global_scale);
    hipLaunchKernelGGL(head_scale_finalize_kernel, dim3(1), dim3(256), 0, st, scale, heads, global_scale);
    return hipGetLastError() == hipSuccess ? IFA_OK : IFA_ERR_HIP;
}

}  // namespace

namespace {
int tokenwise_args(const void *X, int x_dtype, long rows, int d, const signed char *Xq, const float *scale, float scale_mul) {
    if (!X || !Xq || !scale) return IFA_ERR_NULL;
    if (rows <= 0 || d <= 0 || rows > (1L << 40) / d) return IFA_ERR_SHAPE;
    if (x_dtype < IFA_F32 || x_dtype > IFA_BF16) return IFA_ERR_DTYPE;
    if (d != 32 && d != 64 && d != 128 && d != 256 && d != 512) return IFA_ERR_UNSUPPORTED;
    if (!ifa_aligned16(X) || !ifa_aligned16(Xq) || (reinterpret_cast<uintptr_t>(scale) & 3)) return IFA_ERR_UNSUPPORTED;
    if (!(scale_mul > 0.0f) || scale_mul > 3.0e38f) return IFA_ERR_SHAPE;
    return IFA_OK;
}

template <bool HADAMARD>
int tokenwise_launch(const TokenJob &j0, const TokenJob &j1, int jobs, int x_dtype, long rows, int d, unsigned *clear,
                     long clear_words, const HeadJob &hj, hipStream_t st) {
    switch (x_dtype) {
    case IFA_F32: return launch_tokenwise<float, HADAMARD>(j0, j1, jobs, rows, d, clear, clear_words, hj, st);
    case IFA_F16: return launch_tokenwise<__half, HADAMARD>(j0, j1, jobs, rows, d, clear, clear_words, hj, st);
    default: return launch_tokenwise<__hip_bfloat16, HADAMARD>(j0, j1, jobs, rows, d, clear, clear_words, hj, st);
    }
}

template <bool HADAMARD>
int tokenwise_entry(const void *X, int x_dtype, long rows, int d, signed char *Xq, float *scale, float scale_mul,
                    void *hip_stream) {
    const int rc = tokenwise_args(X, x_dtype, rows, d, Xq, scale, scale_mul);
    if (rc != IFA_OK) return rc;
    const TokenJob job = {X, reinterpret_cast<int8_t *>(Xq), scale, scale_mul};
    return tokenwise_launch<HADAMARD>(job, job, 1, x_dtype, rows, d, nullptr, 0, HeadJob{nullptr, nullptr, 0, 0}, static_cast<hipStream_t>(hip_stream));
}

int headwise_args(const void *X, int x_dtype, long heads, long N, int d, const signed char *Xq, const float *scale) {
    if (!X || !Xq || !scale) return IFA_ERR_NULL;
    if (heads <= 0 || N <= 0 || d <= 0 || heads > 65535 || N > (1L << 40) / d / heads) return IFA_ERR_SHAPE;
    if (x_dtype < IFA_F32 || x_dtype > IFA_BF16) return IFA_ERR_DTYPE;
    if ((N * d) % 8 != 0) return IFA_ERR_UNSUPPORTED;
    if (!ifa_aligned16(X) || !ifa_aligned16(Xq) || (reinterpret_cast<uintptr_t>(scale) & 3)) return IFA_ERR_UNSUPPORTED;
    return IFA_OK;
}

int headwise_launch(const void *X, int x_dtype, long heads, long N, int d, signed char *Xq, float *scale, int global_scale,
                    hipStream_t st, bool slots_cleared) {
    int8_t *q = reinterpret_cast<int8_t *>(Xq);
    const int g = global_scale ? 1 : 0;
    switch (x_dtype) {
    case IFA_F32: return launch_headwise<float>(X, heads, N * d, q, scale, g, st, slots_cleared);
    case IFA_F16: return launch_headwise<__half>(X, heads, N * d, q, scale, g, st, slots_cleared);
    default: return launch_headwise<__hip_bfloat16>(X, heads, N * d, q, scale, g, st, slots_cleared);
    }
}
}  // namespace

extern "C" int quantize_tokenwise_ex(const void *X, int x_dtype, long rows, int d, signed char *Xq, float *scale,
                                     float scale_mul, void *hip_stream) {
    return tokenwise_entry<false>(X, x_dtype, rows, d, Xq, scale, scale_mul, hip_stream);
}

extern "C" int quantize_tokenwise_hadamard(const void *X, int x_dtype, long rows, int d, signed char *Xq, float *scale,
                                           float scale_mul, void *hip_stream) {
    return tokenwise_entry<true>(X, x_dtype, rows, d, Xq, scale, scale_mul, hip_stream);
}

extern "C" int quantize_tokenwise(const void *X, int x_dtype, long rows, int d, signed char *Xq, float *scale) {
    return quantize_tokenwise_ex(X, x_dtype, rows, d, Xq, scale, 1.0f, ifa_current_stream());
}

extern "C" int quantize_blockwise(const void *X, int x_dtype, long heads, long N, int d, int block_keys,
                                  signed char *Xq, float *scale, void *hip_stream) {
    if (!X || !Xq || !scale) return IFA_ERR_NULL;
    if (heads <= 0 || N <= 0 || d <= 0 || block_keys <= 0 || heads > 65535 || N > (1L << 40) / d / heads) return IFA_ERR_SHAPE;
    if (x_dtype < IFA_F32 || x_dtype > IFA_BF16) return IFA_ERR_DTYPE;
    if (d % 8 != 0 || static_cast<long>(block_keys) * d > 16384) return IFA_ERR_UNSUPPORTED;
    const long blocks = (N + block_keys - 1) / block_keys;
    if (blocks > 0x7fffffffL) return IFA_ERR_UNSUPPORTED;
    if (!ifa_aligned16(X) || !ifa_aligned16(Xq) || (reinterpret_cast<uintptr_t>(scale) & 3)) return IFA_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    int8_t *q = reinterpret_cast<int8_t *>(Xq);
    const dim3 grid(static_cast<unsigned>(blocks), static_cast<unsigned>(heads)), block(256);
    switch (x_dtype) {
    case IFA_F32: hipLaunchKernelGGL((block_quantize_kernel<float>), grid, block, 0, st, X, N, d, block_keys, q, scale); break;
    case IFA_F16: hipLaunchKernelGGL((block_quantize_kernel<__half>), grid, block, 0, st, X, N, d, block_keys, q, scale); break;
    default: hipLaunchKernelGGL((block_quantize_kernel<__hip_bfloat16>), grid, block, 0, st, X, N, d, block_keys, q, scale); break;
    }
    return hipGetLastError() == hipSuccess ? IFA_OK : IFA_ERR_HIP;
}

extern "C" int quantize_headwise_ex(const void *X, int x_dtype, long heads, long N, int d, signed char *Xq,
                                    float *scale, int global_scale, void *hip_stream) {
    const int rc = headwise_args(X, x_dtype, heads, N, d, Xq, scale);
    if (rc != IFA_OK) return rc;
    return headwise_launch(X, x_dtype, heads, N, d, Xq, scale, global_scale, static_cast<hipStream_t>(hip_stream), false);
}

extern "C" int quantize_headwise(const void *X, int x_dtype, long heads, long N, int d, signed char *Xq,
                                 float *scale, int global_scale) {
    return quantize_headwise_ex(X, x_dtype, heads, N, d, Xq, scale, global_scale, ifa_current_stream());
}

extern "C" int quantize_qk(const void *Q, const void *K, int x_dtype, long rows, int d, signed char *Q_i8, signed char *K_i8,
                           float *s_Q, float *s_K, float s_Q_mul, int hadamard, void *hip_stream) {
    int rc = tokenwise_args(Q, x_dtype, rows, d, Q_i8, s_Q, s_Q_mul);
    if (rc == IFA_OK) rc = tokenwise_args(K, x_dtype, rows, d, K_i8, s_K, 1.0f);
    if (rc != IFA_OK) return rc;
    const TokenJob jq = {Q, reinterpret_cast<int8_t *>(Q_i8), s_Q, s_Q_mul}, jk = {K, reinterpret_cast<int8_t *>(K_i8), s_K, 1.0f};
    const HeadJob none = {nullptr, nullptr, 0, 0};
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    return hadamard ? tokenwise_launch<true>(jq, jk, 2, x_dtype, rows, d, nullptr, 0, none, st)
                    : tokenwise_launch<false>(jq, jk, 2, x_dtype, rows, d, nullptr, 0, none, st);
}

extern "C" int quantize_qkv(const void *Q, const void *K, const void *V, int x_dtype, long heads, long N, int d,
                            signed char *Q_i8, signed char *K_i8, signed char *V_i8, float *s_Q, float *s_K, float *s_V,
                            float s_Q_mul, void *hip_stream) {
    int rc = headwise_args(V, x_dtype, heads, N, d, V_i8, s_V);             // bounds heads * N * d first
    if (rc == IFA_OK) rc = tokenwise_args(Q, x_dtype, heads * N, d, Q_i8, s_Q, s_Q_mul);
    if (rc == IFA_OK) rc = tokenwise_args(K, x_dtype, heads * N, d, K_i8, s_K, 1.0f);
    if (rc != IFA_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const TokenJob jq = {Q, reinterpret_cast<int8_t *>(Q_i8), s_Q, s_Q_mul}, jk = {K, reinterpret_cast<int8_t *>(K_i8), s_K, 1.0f};
    const long per_head = N * d;
    // With enough heads to fill the chip at HEAD_PARTS workgroups each, the absmax pass of V rides in the launch of Q and K
    // (no atomics, no slots to clear) and three launches do the whole preparation; otherwise the general tensor-level
    // path follows the launch of Q and K, which then also clears its slots.
    if (heads >= 32 && per_head >= 64 * HEAD_PARTS) {
        const HeadJob hj = {V, reinterpret_cast<int8_t *>(V_i8), per_head, static_cast<int>(heads)};
        rc = tokenwise_launch<false>(jq, jk, 2, x_dtype, heads * N, d, nullptr, 0, hj, st);
        if (rc != IFA_OK) return rc;
        long bx = (per_head / 8 + 255) / 256;
        const long cap = (256L * 4 + heads - 1) / heads;     // about 4 workgroups per CU in total, as in launch_headwise
        if (bx > cap) bx = cap;
        const dim3 grid(static_cast<unsigned>(bx), static_cast<unsigned>(heads)), tail_grid(static_cast<unsigned>((heads + 63) / 64));
        int8_t *vq = reinterpret_cast<int8_t *>(V_i8);
        switch (x_dtype) {
        case IFA_F32:
            hipLaunchKernelGGL((head_quantize_from_parts_kernel<float>), grid, dim3(256), 0, st, V, per_head, vq);
            hipLaunchKernelGGL((head_tail_finalize_kernel<float>), tail_grid, dim3(64), 0, st, V, per_head, vq, s_V, heads);
            break;
        case IFA_F16:
            hipLaunchKernelGGL((head_quantize_from_parts_kernel<__half>), grid, dim3(256), 0, st, V, per_head, vq);
            hipLaunchKernelGGL((head_tail_finalize_kernel<__half>), tail_grid, dim3(64), 0, st, V, per_head, vq, s_V, heads);
            break;
        default:
            hipLaunchKernelGGL((head_quantize_from_parts_kernel<__hip_bfloat16>), grid, dim3(256), 0, st, V, per_head, vq);
            hipLaunchKernelGGL((head_tail_finalize_kernel<__hip_bfloat16>), tail_grid, dim3(64), 0, st, V, per_head, vq, s_V, heads);
            break;
        }
        return hipGetLastError() == hipSuccess ? IFA_OK : IFA_ERR_HIP;
    }
    // one launch for Q and K, which also clears the slots the absmax pass of V accumulates into
    rc = tokenwise_launch<false>(jq, jk, 2, x_dtype, heads * N, d, reinterpret_cast<unsigned *>(s_V), heads, HeadJob{nullptr, nullptr, 0, 0}, st);
    if (rc != IFA_OK) return rc;
    return headwise_launch(V, x_dtype, heads, N, d, V_i8, s_V, 0, st, true);
}
