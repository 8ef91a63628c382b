// Issue-model micro-benchmark for gfx950: how the matrix pipe (v_mfma_i32_32x32x32_i8), the plain vector ALU and
// the transcendental unit (v_exp_f32) share a SIMD.  It is the evidence behind the instruction schedule of the
// fused attention kernel: every probe is a register-only loop (no memory, no LDS) whose instruction sequence is
// spelled out below, timed three ways -- HIP events around the launch, the shader clock counter (s_memtime) and
// the constant 100 MHz counter (s_memrealtime) inside every wavefront -- so that cycles are real SIMD cycles at
// the clock the probe actually ran at.  Run under `rocprofv3 --pmc ...` the same launches give the instruction
// and busy-cycle counters; each probe is launched exactly twice (warm-up, timed), in the order printed.
//
// A "unit" is what one MFMA is paired with.  Probes:
//   solo    : one instruction kind alone, 32 per unit, on 32 independent registers
//   mix     : per unit 1 MFMA + NV vector instructions of one kind + NE v_exp_f32, issued by the same wavefront
//   split   : one 8-wavefront workgroup per CU; wavefronts 0-3 issue MFMAs only, wavefronts 4-7 vector work only
//             (wavefront w and w + 4 share SIMD w % 4: the hardware id is recorded and printed); each role alone,
//             then both together: if the pipes overlap across wavefronts the together-time is the max, else the sum
//   layers  : W wavefronts per SIMD, each running a program of its own (MFMA only, vector only, exp only, mixes):
//             which pairs of instruction classes overlap across the wavefronts of a SIMD and which take turns
//   phase   : block skeletons made of whole sections (MFMA-only and vector-only stretches), with and without
//             s_setprio around them
//   block   : the register-only skeleton of one key block of the attention kernel (32 MFMA and 496 vector
//             instructions, 64 of them v_exp_f32, in the kernel's own proportions) in several schedules
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>
#include <string>
#include <vector>

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

#define CK(x)                                                                                         \
    do {                                                                                              \
        hipError_t e_ = (x);                                                                          \
        if (e_ != hipSuccess) {                                                                       \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);                     \
            return 1;                                                                                 \
        }                                                                                             \
    } while (0)

struct WaveRec {
    unsigned long long cyc;    // s_memtime ticks spent in the timed loop
    unsigned long long wall;   // s_memrealtime ticks (100 MHz) spent in the timed loop
    unsigned hwid;             // HW_ID register: SIMD in bits 5:4, CU in 11:8, SE in 15:13
    unsigned role;
};
constexpr int MAX_WAVES = 256 * 16 * 4;

enum { FMA1 = 0, FMA3, ADDLIT, MUL2, MAX3, CVTPK, EXP, FMAC, SADU8, NOP_OP, SDWAADD, DOT4, SUBINL, MIN3, PKNORM, PERM, MAX2, CVTI, PKRTZ, PKADD16 };
static const char *OP_NAME[] = {"v_fma_f32 x,x,0.5,0.5", "v_fma_f32 x,x,y,z", "v_add_f32 x,lit,x", "v_mul_f32 x,x,y",
                                "v_max3_f32 x,x,y,z",    "v_cvt_pk_u8_f32 x,y,1,x", "v_exp_f32 x,x", "v_fmac_f32 x,y,z",
                                "v_sad_u8 x,x,0,y", "-", "v_add_f32_sdwa x.b1,y,z", "v_dot4_u32_u8 x,y,z,x", "v_sub_f32 x,inv2pi,x", "v_min3_f32 x,x,y,z", "v_cvt_pknorm_u16_f32 x,x,y", "v_perm_b32 x,x,y,z", "v_max_f32 x,x,y", "v_cvt_f32_i32 x,x",
                                "v_cvt_pkrtz_f16_f32 x,x,y", "v_pk_add_u16 x,x,y"};

#if defined(__HIP_DEVICE_COMPILE__)
template <int OP> __device__ __forceinline__ void vop(float &x, float y, float z) {
    if constexpr (OP == FMA1) asm volatile("v_fma_f32 %0, %0, 0.5, 0.5" : "+v"(x));
    else if constexpr (OP == FMA3) asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(x) : "v"(y), "v"(z));
    else if constexpr (OP == ADDLIT) asm volatile("v_add_f32 %0, 0xcb400000, %0" : "+v"(x));
    else if constexpr (OP == MUL2) asm volatile("v_mul_f32 %0, %0, %1" : "+v"(x) : "v"(y));
    else if constexpr (OP == MAX3) asm volatile("v_max3_f32 %0, %0, %1, %2" : "+v"(x) : "v"(y), "v"(z));
    else if constexpr (OP == CVTPK) asm volatile("v_cvt_pk_u8_f32 %0, %1, 1, %0" : "+v"(x) : "v"(y));
    else if constexpr (OP == EXP) asm volatile("v_exp_f32 %0, %0" : "+v"(x));
    else if constexpr (OP == FMAC) asm volatile("v_fmac_f32 %0, %1, %2" : "+v"(x) : "v"(y), "v"(z));
    else if constexpr (OP == SADU8) asm volatile("v_sad_u8 %0, %0, 0, %1" : "+v"(x) : "v"(y));
    else if constexpr (OP == SDWAADD) asm volatile("v_add_f32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD" : "+v"(x) : "v"(y), "v"(z));
    else if constexpr (OP == DOT4) asm volatile("v_dot4_u32_u8 %0, %1, %2, %0" : "+v"(x) : "v"(y), "v"(z));
    else if constexpr (OP == SUBINL) asm volatile("v_sub_f32 %0, 0.15915494, %0" : "+v"(x));
    else if constexpr (OP == PKNORM) asm volatile("v_cvt_pknorm_u16_f32 %0, %0, %1" : "+v"(x) : "v"(y));
    else if constexpr (OP == PERM) asm volatile("v_perm_b32 %0, %0, %1, %2" : "+v"(x) : "v"(y), "v"(z));
    else if constexpr (OP == MAX2) asm volatile("v_max_f32 %0, %0, %1" : "+v"(x) : "v"(y));
    else if constexpr (OP == CVTI) asm volatile("v_cvt_f32_i32 %0, %0" : "+v"(x));
    else if constexpr (OP == PKRTZ) asm volatile("v_cvt_pkrtz_f16_f32 %0, %0, %1" : "+v"(x) : "v"(y));
    else if constexpr (OP == PKADD16) asm volatile("v_pk_add_u16 %0, %0, %1" : "+v"(x) : "v"(y));
    else if constexpr (OP == MIN3) asm volatile("v_min3_f32 %0, %0, %1, %2" : "+v"(x) : "v"(y), "v"(z));
}
__device__ __forceinline__ void mfma(v16i &c, const v4i &a, const v4i &b) {
    asm volatile("v_mfma_i32_32x32x32_i8 %0, %1, %2, %0" : "+v"(c) : "v"(a), "v"(b));
}
__device__ __forceinline__ unsigned hw_id() {
    return __builtin_amdgcn_s_getreg((15 << 11) | (0 << 6) | 4);   // HW_ID, bits 15:0
}
struct Stamp { unsigned long long c, w; };
__device__ __forceinline__ Stamp stamp() {
    Stamp s;
    s.c = __builtin_readcyclecounter();
    s.w = __builtin_amdgcn_s_memrealtime();
    return s;
}
__device__ __forceinline__ void record(WaveRec *rec, const Stamp &t0, const Stamp &t1, unsigned role) {
    if ((threadIdx.x & 63) == 0) {
        const int w = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
        if (w < MAX_WAVES) rec[w] = WaveRec{t1.c - t0.c, t1.w - t0.w, hw_id(), role};
    }
}
#endif

// The registers every probe works on.  x: 32 independent vector-ALU destinations, e: 16 for v_exp_f32,
// c: 4 accumulators, a / b: MFMA operands.
struct Regs {
    float x[32], e[16], y, z;
    v16i c[4];
    v4i a, b;
};
#if defined(__HIP_DEVICE_COMPILE__)
__device__ __forceinline__ void init(Regs &r, float seed) {
    for (int i = 0; i < 32; ++i) r.x[i] = seed + i * 0.001f + threadIdx.x * 1e-6f;
    for (int i = 0; i < 16; ++i) r.e[i] = -seed - i * 0.01f;
    r.y = 0.999f + seed * 1e-9f;
    r.z = 0.001f + seed * 1e-9f;
    for (int i = 0; i < 4; ++i) r.c[i] = v16i{0};
    r.a = v4i{(int)threadIdx.x, 2, 3, 4};
    r.b = v4i{5, 6, 7, (int)threadIdx.x};
}
__device__ __forceinline__ void finish(Regs &r, float *sink) {
    asm volatile("s_nop 15\n s_nop 15\n s_nop 15" ::: "memory");   // MFMA results have landed
    float s = 0;
    for (int i = 0; i < 32; ++i) s += r.x[i];
    for (int i = 0; i < 16; ++i) s += r.e[i];
    for (int i = 0; i < 4; ++i) s += (float)(r.c[i][0] + r.c[i][7]);
    if (s == 12345.678f) sink[0] = s;
}
#endif

// ---- mix: per unit NM MFMAs (CHAIN: 4 consecutive units accumulate into the same registers, as the k-steps of one
// tile do; otherwise the 4 accumulators rotate), NV instructions of kind OP and NE v_exp_f32.  PHASE = 1: MFMA, its
// vector work, MFMA, ...; PHASE = p: p MFMAs back to back, then the vector work of those p units.
template <int NM, int CHAIN, int OP, int NV, int NE, int PHASE>
__global__ __launch_bounds__(256) void mix_kernel(int iters, WaveRec *rec, float *sink, float seed) {
#if defined(__HIP_DEVICE_COMPILE__)
    Regs r;
    init(r, seed);
    const Stamp t0 = stamp();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int p = 0; p < 16 / PHASE; ++p) {
#pragma unroll
            for (int q = 0; q < PHASE; ++q) {
                const int u = p * PHASE + q;
                if (NM) mfma(r.c[CHAIN ? (u >> 2) & 3 : u & 3], r.a, r.b);
            }
#pragma unroll
            for (int q = 0; q < PHASE; ++q) {
                const int u = p * PHASE + q;
#pragma unroll
                for (int i = 0; i < NV; ++i) vop<OP>(r.x[(u * NV + i) & 31], r.y, r.z);
#pragma unroll
                for (int i = 0; i < NE; ++i) vop<EXP>(r.e[(u * NE + i) & 15], r.y, r.z);
            }
        }
    }
    const Stamp t1 = stamp();
    record(rec, t0, t1, 0);
    finish(r, sink);
#endif
}

// ---- split: 8 wavefronts per workgroup, one workgroup per CU (the LDS array keeps a second one out).
// Wavefronts 0-3 (role 0) issue `ita` x 16 MFMAs, wavefronts 4-7 (role 1) `itb` x 16 x (NV of OP + NE exp).
template <int OP, int NV, int NE>
__global__ __launch_bounds__(512) void split_kernel(int ita, int itb, WaveRec *rec, float *sink, float seed) {
#if defined(__HIP_DEVICE_COMPILE__)
    __shared__ float keep_out[24 * 1024];   // 96 KB: no second workgroup fits the CU's 160 KB
    keep_out[threadIdx.x] = seed;
    __syncthreads();
    Regs r;
    init(r, seed + keep_out[threadIdx.x ^ 1] * 1e-9f);
    const unsigned role = threadIdx.x >> 8;
    const Stamp t0 = stamp();
    if (role == 0) {
        for (int it = 0; it < ita; ++it) {
#pragma unroll
            for (int u = 0; u < 16; ++u) mfma(r.c[u & 3], r.a, r.b);
        }
    } else {
        for (int it = 0; it < itb; ++it) {
#pragma unroll
            for (int u = 0; u < 16; ++u) {
#pragma unroll
                for (int i = 0; i < NV; ++i) vop<OP>(r.x[(u * NV + i) & 31], r.y, r.z);
#pragma unroll
                for (int i = 0; i < NE; ++i) vop<EXP>(r.e[(u * NE + i) & 15], r.y, r.z);
            }
        }
    }
    const Stamp t1 = stamp();
    record(rec, t0, t1, role);
    finish(r, sink);
#endif
}

// ---- block: the skeleton of one key block of the attention kernel per loop iteration, d = 128, B_c = 128:
//   S phase   4 key tiles x (4 chained MFMA; the fp32 work on the previous tile: 16 add-literal, 16 mul, 8 max3)
//   P phase   64 x (fma, exp, cvt_pk_u8) + 16 sad_u8
//   O phase   4 d tiles x (4 chained MFMA; the fold of the previous tile: 16 add-literal, 16 fma)
// SCHED 0: as the kernel issues it (the three phases one after the other)
// SCHED 1: everything spread evenly: after each of the 32 MFMAs 1/32 of all vector work (4 add, 2 mul, 1 max3, 4 fma,
//          2 exp, 2 cvt_pk; sad every second unit)
// SCHED 2: the P phase of the previous block is issued between the MFMAs of the S phase (as if two blocks were
//          in flight: 16 (fma, exp, cvt_pk) after each S MFMA group), the rest as SCHED 0
// SCHED 3: as SCHED 0 but the exps in runs of 16 (SCHED 0: runs of 8) with the fma before and the cvt_pk after each run
// SCHED 4: MFMAs only (32 per block)      SCHED 5: vector work only (SCHED 0 without the MFMAs)
template <int SCHED, int BARRIER>
__global__ __launch_bounds__(256) void block_kernel(int iters, WaveRec *rec, float *sink, float seed) {
#if defined(__HIP_DEVICE_COMPILE__)
    Regs r;
    init(r, seed);
    const Stamp t0 = stamp();
    for (int it = 0; it < iters; ++it) {
        if constexpr (SCHED == 1) {
#pragma unroll
            for (int u = 0; u < 32; ++u) {
                mfma(r.c[(u >> 2) & 3], r.a, r.b);
#pragma unroll
                for (int i = 0; i < 4; ++i) vop<ADDLIT>(r.x[(u * 4 + i) & 7], r.y, r.z);
#pragma unroll
                for (int i = 0; i < 2; ++i) vop<MUL2>(r.x[8 + ((u * 2 + i) & 3)], r.y, r.z);
                vop<MAX3>(r.x[12 + (u & 3)], r.y, r.z);
#pragma unroll
                for (int i = 0; i < 4; ++i) vop<FMA3>(r.x[16 + ((u * 4 + i) & 7)], r.y, r.z);
#pragma unroll
                for (int i = 0; i < 2; ++i) vop<EXP>(r.e[(u * 2 + i) & 15], r.y, r.z);
#pragma unroll
                for (int i = 0; i < 2; ++i) vop<CVTPK>(r.x[24 + ((u * 2 + i) & 3)], r.y, r.z);
                if (u & 1) vop<SADU8>(r.x[28 + ((u >> 1) & 3)], r.y, r.z);
            }
        } else {
            constexpr bool M = SCHED != 5, V = SCHED != 4;
            // 16 (fma, exp, cvt_pk) + 4 sad of the P phase, dependent instructions at least 8 apart
            auto p_quarter = [&]() {
#pragma unroll
                for (int h = 0; h < 2; ++h) {
#pragma unroll
                    for (int i = 0; i < 8; ++i) vop<FMA3>(r.e[8 * h + i], r.y, r.z);
#pragma unroll
                    for (int i = 0; i < 8; ++i) vop<EXP>(r.e[8 * h + i], r.y, r.z);
#pragma unroll
                    for (int i = 0; i < 8; ++i) vop<CVTPK>(r.x[24 + (i & 3)], r.e[8 * h + i], r.z);
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) vop<SADU8>(r.x[28 + i], r.y, r.z);
            };
            // S phase
#pragma unroll
            for (int t = 0; t < 4; ++t) {
#pragma unroll
                for (int k = 0; k < 4; ++k) if (M) mfma(r.c[t & 1], r.a, r.b);
                if (V) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) vop<ADDLIT>(r.x[i], r.y, r.z);
#pragma unroll
                    for (int i = 0; i < 16; ++i) vop<MUL2>(r.x[i], r.y, r.z);
#pragma unroll
                    for (int i = 0; i < 8; ++i) vop<MAX3>(r.x[16 + i], r.y, r.z);
                    if (SCHED == 2) p_quarter();
                }
            }
            // P phase
            if (V && SCHED != 2) {
                if (SCHED == 3) {
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
#pragma unroll
                        for (int i = 0; i < 16; ++i) vop<FMA3>(r.e[i], r.y, r.z);
#pragma unroll
                        for (int i = 0; i < 16; ++i) vop<EXP>(r.e[i], r.y, r.z);
#pragma unroll
                        for (int i = 0; i < 16; ++i) vop<CVTPK>(r.x[16 + (i & 7)], r.e[i], r.z);
#pragma unroll
                        for (int i = 0; i < 4; ++i) vop<SADU8>(r.x[28 + i], r.y, r.z);
                    }
                } else {
#pragma unroll
                    for (int g = 0; g < 4; ++g) p_quarter();
                }
            }
            // O phase
#pragma unroll
            for (int t = 0; t < 4; ++t) {
#pragma unroll
                for (int k = 0; k < 4; ++k) if (M) mfma(r.c[2 + (t & 1)], r.a, r.b);
                if (V) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) vop<ADDLIT>(r.x[i], r.y, r.z);
#pragma unroll
                    for (int i = 0; i < 16; ++i) vop<FMA3>(r.x[16 + (i & 7)], r.x[i], r.z);
                }
            }
        }
        if (BARRIER) __syncthreads();
    }
    const Stamp t1 = stamp();
    record(rec, t0, t1, 0);
    finish(r, sink);
#endif
}

// ---- layers: one workgroup of 256 * W threads per CU (W wavefronts per SIMD; the LDS array keeps a second workgroup
// out); wavefront w runs program PROG[w / 4], so that the W wavefronts sharing a SIMD run W chosen programs side by
// side.  Every layer loops `it[layer]` times over 16 units (0: the layer exits at once) and its mean time is reported.
//   P_MFMA      16 MFMA                                   P_FMA     16 x 12 fma
//   P_EXP       16 x 4 exp                                P_MFMAEXP 16 x (MFMA, 2 exp)
//   P_VMIX      16 x (4 add-literal, 2 mul, 1 max3, 4 fma, 2 cvt_pk_u8, sad every 2nd unit): the kernel's non-exp work
//   P_FULL      16 x (MFMA + VMIX + 2 exp): everything evenly mixed in one wavefront
//   P_ADD / P_MUL / P_MAX3 / P_CVT  16 x 12 of that instruction
enum { P_IDLE = 0, P_MFMA, P_FMA, P_EXP, P_MFMAEXP, P_VMIX, P_FULL, P_ADD, P_MUL, P_MAX3, P_CVT };
static const char *PROG_NAME[] = {"idle", "MFMA", "12 fma", "4 exp", "MFMA+2exp", "vmix(13.5)", "MFMA+vmix+2exp", "12 add-lit", "12 mul", "12 max3", "12 cvt_pk"};

#if defined(__HIP_DEVICE_COMPILE__)
template <int PROG> __device__ __forceinline__ void run_prog(Regs &r, int iters) {
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            if constexpr (PROG == P_MFMA || PROG == P_MFMAEXP || PROG == P_FULL) mfma(r.c[u & 3], r.a, r.b);
            if constexpr (PROG == P_FMA) {
#pragma unroll
                for (int i = 0; i < 12; ++i) vop<FMA1>(r.x[(u * 12 + i) & 31], r.y, r.z);
            }
            if constexpr (PROG == P_ADD) {
#pragma unroll
                for (int i = 0; i < 12; ++i) vop<ADDLIT>(r.x[(u * 12 + i) & 31], r.y, r.z);
            }
            if constexpr (PROG == P_MUL) {
#pragma unroll
                for (int i = 0; i < 12; ++i) vop<MUL2>(r.x[(u * 12 + i) & 31], r.y, r.z);
            }
            if constexpr (PROG == P_MAX3) {
#pragma unroll
                for (int i = 0; i < 12; ++i) vop<MAX3>(r.x[(u * 12 + i) & 31], r.y, r.z);
            }
            if constexpr (PROG == P_CVT) {
#pragma unroll
                for (int i = 0; i < 12; ++i) vop<CVTPK>(r.x[(u * 12 + i) & 31], r.y, r.z);
            }
            if constexpr (PROG == P_VMIX || PROG == P_FULL) {
#pragma unroll
                for (int i = 0; i < 4; ++i) vop<ADDLIT>(r.x[(u * 4 + i) & 7], r.y, r.z);
#pragma unroll
                for (int i = 0; i < 2; ++i) vop<MUL2>(r.x[8 + ((u * 2 + i) & 3)], r.y, r.z);
                vop<MAX3>(r.x[12 + (u & 3)], r.y, r.z);
#pragma unroll
                for (int i = 0; i < 4; ++i) vop<FMA3>(r.x[16 + ((u * 4 + i) & 7)], r.y, r.z);
#pragma unroll
                for (int i = 0; i < 2; ++i) vop<CVTPK>(r.x[24 + ((u * 2 + i) & 3)], r.y, r.z);
                if (u & 1) vop<SADU8>(r.x[28 + ((u >> 1) & 3)], r.y, r.z);
            }
            if constexpr (PROG == P_EXP) {
#pragma unroll
                for (int i = 0; i < 4; ++i) vop<EXP>(r.e[(u * 4 + i) & 15], r.y, r.z);
            }
            if constexpr (PROG == P_MFMAEXP || PROG == P_FULL) {
#pragma unroll
                for (int i = 0; i < 2; ++i) vop<EXP>(r.e[(u * 2 + i) & 15], r.y, r.z);
            }
        }
    }
}
#endif

struct LayerIters { int it[4]; };

template <int W, int PR0, int PR1, int PR2, int PR3>
__global__ __launch_bounds__(256 * W) void layers_kernel(LayerIters li, WaveRec *rec, float *sink, float seed) {
#if defined(__HIP_DEVICE_COMPILE__)
    __shared__ float keep_out[24 * 1024];   // 96 KB: no second workgroup fits the CU's 160 KB
    keep_out[threadIdx.x] = seed;
    __syncthreads();
    Regs r;
    init(r, seed + keep_out[threadIdx.x ^ 1] * 1e-9f);
    const unsigned layer = threadIdx.x >> 8;
    const Stamp t0 = stamp();
    if (layer == 0) run_prog<PR0>(r, li.it[0]);
    else if (layer == 1) run_prog<PR1>(r, li.it[1]);
    else if (layer == 2) run_prog<PR2>(r, li.it[2]);
    else run_prog<PR3>(r, li.it[3]);
    const Stamp t1 = stamp();
    record(rec, t0, t1, layer);
    finish(r, sink);
#endif
}

// ---- phase: block skeletons built from whole sections, W wavefronts per SIMD in one workgroup per CU.
//   STRUCT 0: the kernel's order (as block SCHED 0): MFMA groups of 4 with the fp32 work of the previous tile between
//   STRUCT 1: sections: M1 16 MFMA | V1 64 add-literal, 64 mul, 32 max3 | V2 64 (fma, exp, cvt_pk), 16 sad |
//             M2 16 MFMA | V3 64 add-literal, 64 fma
//   STRUCT 2: as 1, but M2 runs key tile by key tile with the (fma, exp, cvt_pk) of the NEXT tile between its MFMAs:
//             M1 | V1 | P tile 0 | 3 x (4 MFMA with 16 (fma, exp, cvt_pk) + 4 sad among them) | 4 MFMA | V3
//   STRUCT 3: as 1, but V1 is spread over M1 (after each MFMA 4 add, 4 mul, 2 max3) and V3 over M2 (4 add, 4 fma)
//   STRUCT 4: the kernel's S phase (as STRUCT 0), then as STRUCT 2: P tile 0 | M2 with the next tile's exps | V3
//   STRUCT 5: as 2 with two accumulators at a time: P tile 0 | 4 x (2 MFMA (d tiles 0, 1) with 16 (fma, exp, cvt_pk)
//             of the next tile) | 8 MFMA (d tiles 2, 3) | V3
//   STRUCT 6: M1 is only the second half of the S phase (8 MFMA); after V1 one run of 24 MFMAs -- the first half of the
//             NEXT block's S phase, then M2 -- with the (fma, exp, cvt_pk) of P behind the first 20 of them, 3.2 per MFMA
//   PRIO 0: no s_setprio; 1: priority 3 while a section issues MFMAs, 0 otherwise; 2: the reverse; 3: priority 3 in
//   M2 only; 4: in M1 only; 5: as 1 with priority 1 instead of 3
//   LDS_KB: static LDS per workgroup: 96 admits one workgroup per CU, 64 two (then W = 1 and the grid has 2 per CU:
//   the two wavefronts of a SIMD come from different workgroups, as in the attention kernel)
template <int STRUCT, int PRIO, int W, int LDS_KB = 96, int STAG = 0>
__global__ __launch_bounds__(256 * W) void phase_kernel(int iters, WaveRec *rec, float *sink, float seed) {
#if defined(__HIP_DEVICE_COMPILE__)
    __shared__ float keep_out[LDS_KB * 256];
    keep_out[threadIdx.x] = seed;
    __syncthreads();
    Regs r;
    init(r, seed + keep_out[threadIdx.x ^ 1] * 1e-9f);
    auto prio_m = [&](int which) {      // which: 1 = M1 (S phase), 2 = M2 (O phase)
        if (PRIO == 1 || (PRIO == 3 && which == 2) || (PRIO == 4 && which == 1)) __builtin_amdgcn_s_setprio(3);
        if (PRIO == 5) __builtin_amdgcn_s_setprio(1);
        if (PRIO == 2) __builtin_amdgcn_s_setprio(0);
    };
    auto prio_v = [&]() { if (PRIO == 1 || PRIO >= 3) __builtin_amdgcn_s_setprio(0); if (PRIO == 2) __builtin_amdgcn_s_setprio(3); };
    auto p_tile = [&](int h0, int h1) {         // (fma, exp, cvt_pk) for halves h0 .. h1-1 of a 16-key-per-lane tile
#pragma unroll
        for (int h = h0; h < h1; ++h) {
#pragma unroll
            for (int i = 0; i < 8; ++i) vop<FMA3>(r.e[8 * (h & 1) + i], r.y, r.z);
#pragma unroll
            for (int i = 0; i < 8; ++i) vop<EXP>(r.e[8 * (h & 1) + i], r.y, r.z);
#pragma unroll
            for (int i = 0; i < 8; ++i) vop<CVTPK>(r.x[24 + (i & 3)], r.e[8 * (h & 1) + i], r.z);
        }
    };
    const Stamp t0 = stamp();
    for (int it = 0; it < iters; ++it) {
        if constexpr (STRUCT == 0) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                prio_m(1);
#pragma unroll
                for (int k = 0; k < 4; ++k) mfma(r.c[t & 1], r.a, r.b);
                prio_v();
#pragma unroll
                for (int i = 0; i < 16; ++i) vop<ADDLIT>(r.x[i], r.y, r.z);
#pragma unroll
                for (int i = 0; i < 16; ++i) vop<MUL2>(r.x[i], r.y, r.z);
#pragma unroll
                for (int i = 0; i < 8; ++i) vop<MAX3>(r.x[16 + i], r.y, r.z);
            }
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                p_tile(0, 2);
#pragma unroll
                for (int i = 0; i < 4; ++i) vop<SADU8>(r.x[28 + i], r.y, r.z);
            }
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                prio_m(2);
#pragma unroll
                for (int k = 0; k < 4; ++k) mfma(r.c[2 + (t & 1)], r.a, r.b);
                prio_v();
#pragma unroll
                for (int i = 0; i < 16; ++i) vop<ADDLIT>(r.x[i], r.y, r.z);
#pragma unroll
                for (int i = 0; i < 16; ++i) vop<FMA3>(r.x[16 + (i & 7)], r.x[i], r.z);
            }
        } else {
            // M1 (+ V1)
            if constexpr (STRUCT == 4) {
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    prio_m(1);
#pragma unroll
                    for (int k = 0; k < 4; ++k) mfma(r.c[t & 1], r.a, r.b);
                    prio_v();
#pragma unroll
                    for (int i = 0; i < 16; ++i) vop<ADDLIT>(r.x[i], r.y, r.z);
#pragma unroll
                    for (int i = 0; i < 16; ++i) vop<MUL2>(r.x[i], r.y, r.z);
#pragma unroll
                    for (int i = 0; i < 8; ++i) vop<MAX3>(r.x[16 + i], r.y, r.z);
                }
            }
            if (STRUCT != 4) prio_m(1);
#pragma unroll
            for (int u = 0; u < (STRUCT == 4 ? 0 : STRUCT == 6 ? 8 : 16); ++u) {
                mfma(r.c[(u >> 2) & 3], r.a, r.b);
                if (STRUCT == 3) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) vop<ADDLIT>(r.x[(u * 4 + i) & 15], r.y, r.z);
#pragma unroll
                    for (int i = 0; i < 4; ++i) vop<MUL2>(r.x[(u * 4 + i + 8) & 15], r.y, r.z);
#pragma unroll
                    for (int i = 0; i < 2; ++i) vop<MAX3>(r.x[16 + ((u * 2 + i) & 7)], r.y, r.z);
                }
            }
            prio_v();
            if (STRUCT != 3 && STRUCT != 4) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) vop<ADDLIT>(r.x[i], r.y, r.z);
#pragma unroll
                    for (int i = 0; i < 16; ++i) vop<MUL2>(r.x[i], r.y, r.z);
#pragma unroll
                    for (int i = 0; i < 8; ++i) vop<MAX3>(r.x[16 + i], r.y, r.z);
                }
            }
            if (STAG == 3 && (threadIdx.x >> 8) == 1) __builtin_amdgcn_s_barrier();   // half a block apart
            // V2 / M2
            if (STRUCT == 5) {
                p_tile(0, 2);
#pragma unroll
                for (int i = 0; i < 4; ++i) vop<SADU8>(r.x[28 + i], r.y, r.z);
                prio_m(2);
#pragma unroll
                for (int t = 0; t < 4; ++t) {
#pragma unroll
                    for (int k = 0; k < 2; ++k) {
                        mfma(r.c[k], r.a, r.b);
                        if (t < 3) {            // half of the next tile's P work after each MFMA
#pragma unroll
                            for (int i = 0; i < 8; ++i) vop<FMA3>(r.e[8 * k + i], r.y, r.z);
#pragma unroll
                            for (int i = 0; i < 8; ++i) vop<EXP>(r.e[8 * k + i], r.y, r.z);
#pragma unroll
                            for (int i = 0; i < 8; ++i) vop<CVTPK>(r.x[24 + (i & 3)], r.e[8 * (k ^ 1) + i], r.z);
                            vop<SADU8>(r.x[28 + k], r.y, r.z);
                            vop<SADU8>(r.x[30 + k], r.y, r.z);
                        }
                    }
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) mfma(r.c[2 + (u >> 2)], r.a, r.b);
                prio_v();
            } else if (STRUCT == 6) {
                // 8 MFMAs of the NEXT block's S phase, then the 16 of this block's O phase: one run of 24 MFMAs; the 64
                // (fma, exp, cvt_pk) of P go behind the first 20 of them, 3.2 per MFMA (P tile t is complete before MFMA 8 + 4 t)
                prio_m(2);
#pragma unroll
                for (int u = 0; u < 24; ++u) {
                    mfma(r.c[(u >> 2) & 3], r.a, r.b);
                    if (u < 20) {
                        const int lo = (u * 16 + 4) / 5, hi = ((u + 1) * 16 + 4) / 5;
#pragma unroll
                        for (int e = lo; e < hi; ++e) vop<FMA3>(r.e[e & 15], r.y, r.z);
#pragma unroll
                        for (int e = lo; e < hi; ++e) vop<EXP>(r.e[e & 15], r.y, r.z);
#pragma unroll
                        for (int e = lo; e < hi; ++e) vop<CVTPK>(r.x[24 + (e & 3)], r.e[(e + 8) & 15], r.z);
                        if (u < 16) vop<SADU8>(r.x[28 + (u & 3)], r.y, r.z);
                    }
                }
                prio_v();
            } else if (STRUCT == 2 || STRUCT == 4) {
                p_tile(0, 2);
#pragma unroll
                for (int i = 0; i < 4; ++i) vop<SADU8>(r.x[28 + i], r.y, r.z);
                prio_m(2);
#pragma unroll
                for (int t = 0; t < 4; ++t) {
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        mfma(r.c[k], r.a, r.b);
                        if (t < 3) {            // a quarter of the next tile's P work after each MFMA
#pragma unroll
                            for (int i = 0; i < 4; ++i) vop<FMA3>(r.e[4 * k + i], r.y, r.z);
#pragma unroll
                            for (int i = 0; i < 4; ++i) vop<EXP>(r.e[4 * k + i], r.y, r.z);
#pragma unroll
                            for (int i = 0; i < 4; ++i) vop<CVTPK>(r.x[24 + i], r.e[4 * ((k + 3) & 3) + i], r.z);
                            vop<SADU8>(r.x[28 + k], r.y, r.z);
                        }
                    }
                }
                prio_v();
            } else {
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    p_tile(0, 2);
#pragma unroll
                    for (int i = 0; i < 4; ++i) vop<SADU8>(r.x[28 + i], r.y, r.z);
                }
                prio_m(2);
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    mfma(r.c[(u >> 2) & 3], r.a, r.b);
                    if (STRUCT == 3) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) vop<ADDLIT>(r.x[(u * 4 + i) & 15], r.y, r.z);
#pragma unroll
                        for (int i = 0; i < 4; ++i) vop<FMA3>(r.x[16 + ((u * 4 + i) & 7)], r.x[(u * 4 + i + 8) & 15], r.z);
                    }
                }
                prio_v();
            }
            // STAG 1: the two wavefronts of a SIMD (w and w + 4) meet one workgroup barrier per block at DIFFERENT points of
            // their program -- wavefronts 4-7 in front of V3, wavefronts 0-3 behind it -- which holds them one section apart;
            // STAG 2: same barrier point for all (behind V3): held in the same section
            if (STAG == 1 && (threadIdx.x >> 8) == 1) __builtin_amdgcn_s_barrier();
            // V3
            if (STRUCT != 3) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) vop<ADDLIT>(r.x[i], r.y, r.z);
#pragma unroll
                    for (int i = 0; i < 16; ++i) vop<FMA3>(r.x[16 + (i & 7)], r.x[i], r.z);
                }
            }
            if (((STAG == 1 || STAG == 3) && (threadIdx.x >> 8) == 0) || STAG == 2) __builtin_amdgcn_s_barrier();
        }
    }
    const Stamp t1 = stamp();
    record(rec, t0, t1, threadIdx.x >> 8);
    finish(r, sink);
#endif
}

// ---- host --------------------------------------------------------------------------------------------------------
struct Result { float ms; double cyc, wall; int waves; double cyc_role[4], wall_role[4]; int n_role[4]; unsigned simd_w0, simd_w4; };

static WaveRec *g_rec;
static float *g_sink;
static std::vector<WaveRec> g_host(MAX_WAVES);
static int g_dispatch = 0;

template <typename L> static Result run(L launch, int waves) {
    hipEvent_t a, b;
    (void)hipEventCreate(&a);
    (void)hipEventCreate(&b);
    launch();
    (void)hipDeviceSynchronize();
    (void)hipMemset(g_rec, 0, sizeof(WaveRec) * MAX_WAVES);
    (void)hipEventRecord(a);
    launch();
    (void)hipEventRecord(b);
    (void)hipEventSynchronize(b);
    g_dispatch += 2;
    Result r{};
    (void)hipEventElapsedTime(&r.ms, a, b);
    (void)hipMemcpy(g_host.data(), g_rec, sizeof(WaveRec) * waves, hipMemcpyDeviceToHost);
    r.waves = waves;
    for (int i = 0; i < waves; ++i) {
        const WaveRec &w = g_host[i];
        r.cyc += (double)w.cyc / waves;
        r.wall += (double)w.wall / waves;
        const int ro = w.role & 3;
        r.cyc_role[ro] += (double)w.cyc;
        r.wall_role[ro] += (double)w.wall;
        r.n_role[ro]++;
    }
    for (int ro = 0; ro < 4; ++ro)
        if (r.n_role[ro]) { r.cyc_role[ro] /= r.n_role[ro]; r.wall_role[ro] /= r.n_role[ro]; }
    r.simd_w0 = (g_host[0].hwid >> 4) & 3;
    r.simd_w4 = waves > 4 ? (g_host[4].hwid >> 4) & 3 : 9;
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(b);
    return r;
}

static const char *g_only = nullptr;
static bool want(const char *section) { return !g_only || strstr(section, g_only); }

int main(int argc, char **argv) {
    for (int i = 1; i + 1 < argc; ++i)
        if (!strcmp(argv[i], "--only")) g_only = argv[i + 1];
    int dev = 0;
    hipDeviceProp_t prop;
    CK(hipGetDeviceProperties(&prop, dev));
    const int CU = prop.multiProcessorCount;
    printf("device %s, %d CUs, nominal %d MHz; every probe is launched twice (warm-up, timed); dispatch ids are 1-based launch order\n",
           prop.gcnArchName, CU, prop.clockRate / 1000);
    printf("clk = s_memtime ticks per wavefront / (s_memrealtime ticks / 100 MHz): the shader clock the probe ran at, if s_memtime counts shader cycles\n");
    CK(hipMalloc(&g_rec, sizeof(WaveRec) * MAX_WAVES));
    CK(hipMalloc(&g_sink, 64));
    const int iters = 2000;

    // cycles per unit per SIMD: each SIMD runs `wps` wavefronts concurrently, each doing iters * units_per_iter units
    auto line = [&](const char *name, int wps, const Result &r, double units_per_wave) {
        const double mhz = r.wall > 0 ? r.cyc / r.wall * 100.0 : 0.0;
        const double ev_cyc = r.ms * 1e-3 * mhz * 1e6 / (units_per_wave * wps);      // launch time in cycles at the measured clock
        const double wv_cyc = r.cyc / (units_per_wave * wps);                        // in-wave cycle counter
        const double wall_ns = r.wall * 10.0 / (units_per_wave * wps);
        printf("[d%3d] %-58s wps %d | %8.3f ms | clk %6.0f MHz | per unit per SIMD: %7.2f cyc (events), %7.2f cyc (s_memtime), %7.2f ns\n",
               g_dispatch, name, wps, r.ms, mhz, ev_cyc, wv_cyc, wall_ns);
        fflush(stdout);
    };

#define MIX(NM, CHAIN, OP, NV, NE, PHASE, WPS)                                                                    \
    {                                                                                                             \
        const Result r = run([&] { hipLaunchKernelGGL((mix_kernel<NM, CHAIN, OP, NV, NE, PHASE>), WPS * CU, 256, 0, 0, iters, g_rec, g_sink, 0.5f); }, \
                             WPS * CU * 4);                                                                       \
        char nm[128];                                                                                             \
        snprintf(nm, sizeof nm, "%s%s%d x %s + %d exp%s", NM ? "MFMA" : "no MFMA", CHAIN ? " (chained) + " : " + ", NV, OP_NAME[OP], NE, \
                 PHASE > 1 ? (PHASE == 4 ? " | phases of 4" : " | phases of 16") : "");                           \
        line(nm, WPS, r, iters * 16.0);                                                                           \
    }

    if (want("solo")) {
        printf("\n== solo: 32 instructions of one kind per unit (cycles per unit / 32 = cycles per instruction per SIMD)\n");
#define SOLO(OP) MIX(0, 0, OP, 32, 0, 1, 1) MIX(0, 0, OP, 32, 0, 1, 2) MIX(0, 0, OP, 32, 0, 1, 4)
        SOLO(FMA1) SOLO(FMA3) SOLO(ADDLIT) SOLO(MUL2) SOLO(MAX3) SOLO(CVTPK) SOLO(FMAC) SOLO(SADU8) SOLO(SDWAADD) SOLO(DOT4) SOLO(SUBINL) SOLO(PKNORM) SOLO(PERM) SOLO(MAX2) SOLO(CVTI) SOLO(PKRTZ) SOLO(PKADD16)
        MIX(0, 0, NOP_OP, 0, 16, 1, 1) MIX(0, 0, NOP_OP, 0, 16, 1, 2) MIX(0, 0, NOP_OP, 0, 16, 1, 4)
        printf("   (last three lines: 16 v_exp_f32 per unit)\n");
    }
    if (want("mfma")) {
        printf("\n== mfma: v_mfma_i32_32x32x32_i8 alone, one per unit (32 cycles is the datasheet rate)\n");
        MIX(1, 0, NOP_OP, 0, 0, 1, 1) MIX(1, 0, NOP_OP, 0, 0, 1, 2) MIX(1, 0, NOP_OP, 0, 0, 1, 4)
        MIX(1, 1, NOP_OP, 0, 0, 1, 1) MIX(1, 1, NOP_OP, 0, 0, 1, 2)
    }
    if (want("mix")) {
        printf("\n== mix: one MFMA per unit plus vector work issued by the same wavefront\n");
        MIX(1, 0, FMA1, 4, 0, 1, 2) MIX(1, 0, FMA1, 8, 0, 1, 2) MIX(1, 0, FMA1, 12, 0, 1, 2) MIX(1, 0, FMA1, 16, 0, 1, 2) MIX(1, 0, FMA1, 24, 0, 1, 2)
        MIX(1, 0, FMA3, 8, 0, 1, 2) MIX(1, 0, FMA3, 16, 0, 1, 2)
        MIX(1, 0, ADDLIT, 8, 0, 1, 2) MIX(1, 0, ADDLIT, 16, 0, 1, 2)
        MIX(1, 0, MUL2, 8, 0, 1, 2) MIX(1, 0, MUL2, 16, 0, 1, 2)
        MIX(1, 0, NOP_OP, 0, 1, 1, 2) MIX(1, 0, NOP_OP, 0, 2, 1, 2) MIX(1, 0, NOP_OP, 0, 3, 1, 2) MIX(1, 0, NOP_OP, 0, 4, 1, 2) MIX(1, 0, NOP_OP, 0, 6, 1, 2)
        MIX(1, 0, FMA1, 12, 2, 1, 2) MIX(1, 0, FMA1, 12, 2, 1, 4)
        MIX(0, 0, FMA1, 12, 2, 1, 2)
        MIX(1, 1, FMA1, 12, 2, 1, 2)
        MIX(1, 1, FMA1, 12, 2, 4, 2) MIX(1, 1, FMA1, 12, 2, 16, 2)
        MIX(1, 0, FMA1, 8, 0, 1, 1) MIX(1, 0, FMA1, 16, 0, 1, 1) MIX(1, 0, FMA1, 8, 0, 1, 4) MIX(1, 0, FMA1, 16, 0, 1, 4)
    }
    if (want("split")) {
        printf("\n== split: one 8-wavefront workgroup per CU; wavefronts 0-3 MFMA only (role 0), wavefronts 4-7 vector only (role 1)\n");
        printf("   per-role time = mean s_memrealtime span of that role's wavefronts, in ns per 16-unit iteration\n");
        auto split_line = [&](const char *name, const Result &r, int ita, int itb) {
            const double mhz = r.wall > 0 ? r.cyc / r.wall * 100.0 : 0.0;
            printf("[d%3d] %-46s | %8.3f ms | clk %6.0f MHz | SIMD of wavefront 0 / 4: %u / %u | MFMA role: %8.1f ns/iter%s | vector role: %8.1f ns/iter%s\n",
                   g_dispatch, name, r.ms, mhz, r.simd_w0, r.simd_w4, ita ? r.wall_role[0] * 10.0 / ita : 0.0, ita ? "" : " (idle)",
                   itb ? r.wall_role[1] * 10.0 / itb : 0.0, itb ? "" : " (idle)");
            fflush(stdout);
        };
#define SPLIT(OP, NV, NE, ITA, ITB, LABEL)                                                                                          \
    {                                                                                                                             \
        const Result r = run([&] { hipLaunchKernelGGL((split_kernel<OP, NV, NE>), CU, 512, 0, 0, ITA, ITB, g_rec, g_sink, 0.5f); }, CU * 8); \
        split_line(LABEL, r, ITA, ITB);                                                                                           \
    }
        // 16 MFMAs = 512 cycles per iteration; 16 x 12 fma at ~2.7 = ~520 cycles per iteration
        SPLIT(FMA1, 12, 0, iters, 0, "MFMA alone")
        SPLIT(FMA1, 12, 0, 0, iters, "12 fma per unit alone")
        SPLIT(FMA1, 12, 0, iters, iters, "MFMA || 12 fma per unit")
        SPLIT(FMA3, 12, 0, 0, iters, "12 fma(3 src) per unit alone")
        SPLIT(FMA3, 12, 0, iters, iters, "MFMA || 12 fma(3 src) per unit")
        SPLIT(NOP_OP, 0, 4, 0, iters, "4 exp per unit alone")
        SPLIT(NOP_OP, 0, 4, iters, iters, "MFMA || 4 exp per unit")
        SPLIT(FMA1, 8, 2, 0, iters, "8 fma + 2 exp per unit alone")
        SPLIT(FMA1, 8, 2, iters, iters, "MFMA || 8 fma + 2 exp per unit")
        SPLIT(MUL2, 12, 0, 0, iters, "12 mul per unit alone")
        SPLIT(MUL2, 12, 0, iters, iters, "MFMA || 12 mul per unit")
    }
    if (want("layers")) {
        printf("\n== layers: W wavefronts per SIMD, each running its own program (one workgroup of 256 W threads per CU)\n");
        printf("   per layer: ns and shader cycles per unit (1 unit = what the program lists once; 16 units per loop iteration)\n");
        auto layers_line = [&](int W, const int *progs, const LayerIters &li, const Result &r) {
            const double mhz = r.wall > 0 ? r.cyc / r.wall * 100.0 : 0.0;
            printf("[d%3d] W=%d | %8.3f ms | clk %6.0f MHz |", g_dispatch, W, r.ms, mhz);
            for (int l = 0; l < W; ++l) {
                if (li.it[l]) printf(" %-14s %6.2f ns %6.1f cyc |", PROG_NAME[progs[l]], r.wall_role[l] * 10.0 / (li.it[l] * 16.0), r.cyc_role[l] / (li.it[l] * 16.0));
                else printf(" %-14s   (off)            |", PROG_NAME[progs[l]]);
            }
            printf("\n");
            fflush(stdout);
        };
#define LAYERS(W, A, B, C, D, IA, IB, IC, ID)                                                                                   \
    {                                                                                                                           \
        const LayerIters li = {{IA, IB, IC, ID}};                                                                               \
        const int progs[4] = {A, B, C, D};                                                                                      \
        const Result r = run([&] { hipLaunchKernelGGL((layers_kernel<W, A, B, C, D>), CU, 256 * W, 0, 0, li, g_rec, g_sink, 0.5f); }, CU * 4 * W); \
        layers_line(W, progs, li, r);                                                                                           \
    }
        const int n = iters;
        // each program alone (one wavefront per SIMD active)
        LAYERS(2, P_MFMA, P_IDLE, P_IDLE, P_IDLE, n, 0, 0, 0)
        LAYERS(2, P_MFMAEXP, P_IDLE, P_IDLE, P_IDLE, n, 0, 0, 0)
        LAYERS(2, P_VMIX, P_IDLE, P_IDLE, P_IDLE, n, 0, 0, 0)
        LAYERS(2, P_FULL, P_IDLE, P_IDLE, P_IDLE, n, 0, 0, 0)
        LAYERS(2, P_EXP, P_IDLE, P_IDLE, P_IDLE, n, 0, 0, 0)
        LAYERS(2, P_FMA, P_IDLE, P_IDLE, P_IDLE, n, 0, 0, 0)
        // two wavefronts per SIMD
        LAYERS(2, P_MFMA, P_VMIX, P_IDLE, P_IDLE, 2 * n, n, 0, 0)
        LAYERS(2, P_MFMAEXP, P_VMIX, P_IDLE, P_IDLE, 2 * n, n, 0, 0)
        LAYERS(2, P_MFMA, P_EXP, P_IDLE, P_IDLE, n, n, 0, 0)
        LAYERS(2, P_MFMA, P_FMA, P_IDLE, P_IDLE, 2 * n, n, 0, 0)
        LAYERS(2, P_MFMA, P_ADD, P_IDLE, P_IDLE, 2 * n, n, 0, 0)
        LAYERS(2, P_MFMA, P_MUL, P_IDLE, P_IDLE, 2 * n, n, 0, 0)
        LAYERS(2, P_MFMA, P_MAX3, P_IDLE, P_IDLE, 2 * n, n, 0, 0)
        LAYERS(2, P_MFMA, P_CVT, P_IDLE, P_IDLE, 2 * n, n, 0, 0)
        LAYERS(2, P_VMIX, P_VMIX, P_IDLE, P_IDLE, n, n, 0, 0)
        LAYERS(2, P_FMA, P_FMA, P_IDLE, P_IDLE, n, n, 0, 0)
        LAYERS(2, P_FULL, P_FULL, P_IDLE, P_IDLE, n, n, 0, 0)
        LAYERS(2, P_MFMA, P_MFMA, P_IDLE, P_IDLE, n, n, 0, 0)
        LAYERS(2, P_EXP, P_FMA, P_IDLE, P_IDLE, n, n, 0, 0)
        // three wavefronts per SIMD: the vector port saturated by two wavefronts, one more issuing MFMAs
        LAYERS(3, P_MFMA, P_FMA, P_FMA, P_IDLE, 2 * n, n, n, 0)
        LAYERS(3, P_IDLE, P_FMA, P_FMA, P_IDLE, 0, n, n, 0)
        LAYERS(3, P_MFMA, P_VMIX, P_VMIX, P_IDLE, 2 * n, n, n, 0)
        LAYERS(3, P_IDLE, P_VMIX, P_VMIX, P_IDLE, 0, n, n, 0)
        LAYERS(3, P_MFMAEXP, P_VMIX, P_VMIX, P_IDLE, 2 * n, n, n, 0)
        LAYERS(3, P_FULL, P_FULL, P_FULL, P_IDLE, n, n, n, 0)
        // four wavefronts per SIMD
        LAYERS(4, P_MFMAEXP, P_VMIX, P_VMIX, P_VMIX, 3 * n, n, n, n)
        LAYERS(4, P_MFMAEXP, P_MFMAEXP, P_VMIX, P_VMIX, n, n, n, n)
        LAYERS(4, P_FULL, P_FULL, P_FULL, P_FULL, n, n, n, n)
        LAYERS(4, P_MFMA, P_FMA, P_FMA, P_FMA, 3 * n, n, n, n)
    }
    if (want("phase")) {
        printf("\n== phase: block skeletons built from whole sections; one workgroup of 256 W threads per CU (W wavefronts per SIMD)\n");
        printf("   per block per SIMD = launch time / (iterations x W); per layer = that layer's own mean time per block\n");
        const int bit = 1500;
        static const char *STRUCT_NAME[] = {"kernel order (MFMA groups of 4, fp32 work between)", "sections M1 | V1 | V2 | M2 | V3",
                                            "sections, exps of the next P tile inside M2", "V1 spread over M1, V3 over M2, V2 apart",
                                            "kernel-order S phase, then exps inside M2", "exps inside M2, two accumulators at a time",
                                            "half of the next S phase in front of M2, exps under both"};
        static const char *PRIO_NAME[] = {"no setprio", "prio 3 in MFMA sections", "prio 3 in vector sections", "prio 3 in M2 only", "prio 3 in M1 only", "prio 1 in MFMA sections"};
        auto phase_line = [&](int st, int pr, int W, const Result &r) {
            const double mhz = r.wall > 0 ? r.cyc / r.wall * 100.0 : 0.0;
            const double ev_cyc = r.ms * 1e-3 * mhz * 1e6 / (bit * (double)W);
            printf("[d%3d] %-52s | %-26s | W=%d | %8.3f ms | clk %6.0f MHz | per block per SIMD %7.1f cyc -> MFMA busy %5.1f %% | layers:",
                   g_dispatch, STRUCT_NAME[st], PRIO_NAME[pr], W, r.ms, mhz, ev_cyc, 100.0 * 1024.0 / ev_cyc);
            for (int l = 0; l < W; ++l) printf(" %7.1f", r.cyc_role[l] / bit);
            printf(" cyc\n");
            fflush(stdout);
        };
#define PHASE(ST, PR, W)                                                                                                        \
    {                                                                                                                           \
        const Result r = run([&] { hipLaunchKernelGGL((phase_kernel<ST, PR, W>), CU, 256 * W, 0, 0, bit, g_rec, g_sink, 0.5f); }, CU * 4 * W); \
        phase_line(ST, PR, W, r);                                                                                               \
    }
        PHASE(0, 0, 1) PHASE(1, 0, 1) PHASE(2, 0, 1) PHASE(3, 0, 1)
        PHASE(0, 0, 2) PHASE(0, 1, 2) PHASE(0, 2, 2)
        PHASE(1, 0, 2) PHASE(1, 1, 2) PHASE(1, 2, 2)
        PHASE(2, 0, 2) PHASE(2, 1, 2) PHASE(2, 2, 2)
        PHASE(3, 0, 2) PHASE(3, 1, 2) PHASE(3, 2, 2)
        PHASE(1, 0, 3) PHASE(1, 1, 3) PHASE(2, 1, 3)
        PHASE(1, 0, 4) PHASE(1, 1, 4) PHASE(2, 1, 4)
        PHASE(2, 3, 2) PHASE(2, 4, 2) PHASE(2, 5, 2)
        PHASE(4, 0, 2) PHASE(4, 1, 2) PHASE(4, 3, 2)
        PHASE(5, 0, 2) PHASE(5, 1, 2) PHASE(5, 3, 2)
        PHASE(6, 0, 2) PHASE(6, 1, 2) PHASE(6, 3, 2)
        printf("   one 8-wavefront workgroup, one barrier per block: same point for all wavefronts / wavefronts 4-7 one section ahead of it (in front of V3) / half a block ahead (in front of M2):\n");
#define PHASESTAG(ST, PR, SG)                                                                                                    \
    {                                                                                                                           \
        const Result r = run([&] { hipLaunchKernelGGL((phase_kernel<ST, PR, 2, 96, SG>), CU, 512, 0, 0, bit, g_rec, g_sink, 0.5f); }, CU * 8); \
        printf("   stagger %d: ", SG);                                                                                         \
        phase_line(ST, PR, 2, r);                                                                                               \
    }
        PHASESTAG(1, 0, 2) PHASESTAG(1, 0, 1) PHASESTAG(1, 0, 3)
        PHASESTAG(2, 0, 2) PHASESTAG(2, 0, 1) PHASESTAG(2, 0, 3)
        PHASESTAG(2, 3, 2) PHASESTAG(2, 3, 1) PHASESTAG(2, 3, 3)
        PHASESTAG(1, 3, 1) PHASESTAG(1, 1, 1) PHASESTAG(2, 1, 1)
        printf("   two 4-wavefront workgroups per CU (64 KB of LDS each) instead of one 8-wavefront workgroup:\n");
#define PHASE2WG(ST, PR)                                                                                                        \
    {                                                                                                                           \
        const Result r = run([&] { hipLaunchKernelGGL((phase_kernel<ST, PR, 1, 64>), 2 * CU, 256, 0, 0, bit, g_rec, g_sink, 0.5f); }, CU * 8); \
        Result r2 = r;                                                                                                          \
        r2.ms = r.ms;                                                                                                           \
        phase_line(ST, PR, 2, r2);                                                                                              \
    }
        PHASE2WG(0, 0) PHASE2WG(2, 0) PHASE2WG(2, 1) PHASE2WG(2, 3) PHASE2WG(4, 1) PHASE2WG(4, 3) PHASE2WG(5, 1) PHASE2WG(6, 1) PHASE2WG(6, 3)
    }
    if (want("block")) {
        printf("\n== block: skeleton of one key block of the attention kernel per iteration (32 MFMA = 1024 cycles at the datasheet rate)\n");
        const int bit = 1500;
        auto block_line = [&](const char *name, int wps, const Result &r) {
            const double mhz = r.wall > 0 ? r.cyc / r.wall * 100.0 : 0.0;
            const double ev_cyc = r.ms * 1e-3 * mhz * 1e6 / (bit * (double)wps);
            printf("[d%3d] %-66s wps %d | %8.3f ms | clk %6.0f MHz | per block per SIMD: %7.1f cyc (events), %7.1f cyc (s_memtime) -> MFMA busy %5.1f %%\n",
                   g_dispatch, name, wps, r.ms, mhz, ev_cyc, r.cyc / (bit * (double)wps), 100.0 * 1024.0 / ev_cyc);
            fflush(stdout);
        };
#define BLOCK(SCHED, BAR, WPS, LABEL)                                                                                               \
    {                                                                                                                             \
        const Result r = run([&] { hipLaunchKernelGGL((block_kernel<SCHED, BAR>), WPS * CU, 256, 0, 0, bit, g_rec, g_sink, 0.5f); }, WPS * CU * 4); \
        block_line(LABEL, WPS, r);                                                                                                \
    }
        BLOCK(4, 0, 2, "MFMAs only (32 per block)")
        BLOCK(5, 0, 2, "vector work only (496 per block, 64 of them exp)")
        BLOCK(0, 0, 2, "kernel order: S phase, P phase, O phase")
        BLOCK(0, 1, 2, "kernel order + workgroup barrier per block")
        BLOCK(1, 0, 2, "evenly spread: 1/32 of the vector work after every MFMA")
        BLOCK(2, 0, 2, "P phase of the previous block inside the S phase")
        BLOCK(3, 0, 2, "kernel order, exps in runs of 16")
        BLOCK(0, 0, 1, "kernel order, 1 wavefront per SIMD")
        BLOCK(1, 0, 1, "evenly spread, 1 wavefront per SIMD")
        BLOCK(0, 0, 3, "kernel order, 3 wavefronts per SIMD")
        BLOCK(0, 0, 4, "kernel order, 4 wavefronts per SIMD")
        BLOCK(1, 0, 4, "evenly spread, 4 wavefronts per SIMD")
        BLOCK(2, 0, 4, "P phase inside the S phase, 4 wavefronts per SIMD")
    }
    printf("\ndone: %d dispatches\n", g_dispatch);
    return 0;
}
