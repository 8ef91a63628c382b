// Device-side helpers shared by the attention kernels of libintfa.so (gfx950 only; not part of the C ABI).
#ifndef INTFA_DEVICE_H
#define INTFA_DEVICE_H

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <hip/hip_bf16.h>
#include <stdint.h>

namespace ifa_dev {

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));

#define LDS_AS __attribute__((address_space(3)))
#define GLOBAL_AS __attribute__((address_space(1)))
typedef LDS_AS int8_t *lds_ptr;

constexpr int BR = 128;       // query rows per workgroup
constexpr int THREADS = 256;  // 4 wavefronts x 32 query rows
constexpr float LOG2E = 1.44269504088896340736f;

// The integer GEMMs start their accumulators at the bit pattern of 1.5 * 2^23 instead of 0: an int32 sum s with
// |s| < 2^22 then reads, as a float, exactly 1.5 * 2^23 + s, and one fp32 subtraction replaces v_cvt_f32_i32 (which
// costs twice a subtraction on this chip).  |Q K^T| <= 128 * 128 * 128 = 2^21 and |P V| <= 128 * 127 * 128 < 2^21.
constexpr int ACC_BIAS_I = 0x4B400000;
constexpr float ACC_BIAS_F = 12582912.0f;
// The INT8 kernel goes one step further: its accumulators start at the bit pattern of 1 / (2 pi), 0x3E22F983, which the
// MFMA takes as an INLINE constant (no registers hold it).  That float sits 2291075 steps above the bottom of its
// binade [2^-3, 2^-2), where one step is 2^-26: a sum s in [-2291075, 6097532] reads as 1 / (2 pi) + s 2^-26 exactly,
// and (1 / (2 pi)) - acc = -s 2^-26 is one v_sub_f32 with an inline constant operand (4-byte encoding).
// |Q K^T| <= 128^3 = 2097152 and |P V| <= 127 * 128 * 128 = 2080768 for B_c = 128 both fit.
constexpr int ACC_START_I = 0x3E22F983;
constexpr float ACC_START_F = 0.15915494309189532f;   // rounds to 0x3E22F983
constexpr float ACC_UNIT = 67108864.0f;               // 2^26: accumulator steps per unit of the float view

// Heads an XCD works on at a time (measured on MI355X over group sizes 1 .. 32; the default 4 is never far off).
// Without the mask every workgroup of a head walks all of its K and V, and what a group streams at a time should fit
// the XCD's 4 MB L2: 4 MB / (K + V bytes of a head), between 1 and 4 (long sequences run 2-3 % faster with 1 or 2
// heads than with 4).  Under the mask the query blocks of a head are uneven and run heaviest first, and more heads
// per group even the 64 workgroup slots of an XCD out better: 8 heads when their K and V still fit the L2 and a head
// has at least 10 query blocks (N = 2048, d = 128: +5 % over 4; no gain below).  Once 8 heads exceed the L2 (N = 4096)
// 8 per group still measures 2-4 % faster, but the XCDs then fetch K and V from memory twice over (FETCH_SIZE 1.99 x
// the algorithmic reads against 1.19 x): not taken.
constexpr int HEAD_GROUP = 4;
inline int head_group_for(bool causal, long kv_bytes_per_head, int T_r) {
    const long fit = (4L << 20) / (kv_bytes_per_head > 0 ? kv_bytes_per_head : 1);
    if (causal) return (fit >= 8 && T_r >= 10) ? 8 : HEAD_GROUP;
    return static_cast<int>(fit < 1 ? 1 : (fit > HEAD_GROUP ? HEAD_GROUP : fit));
}

// Workgroups go round-robin over the 8 XCDs by linear id.  All query blocks of a head run on one XCD,
// so its K/V stay in that XCD's L2; an XCD takes its heads `head_group` at a time and, inside a group,
// the query blocks of all its heads in the order `qord` = 0, 1, ... (a causal kernel maps qord 0 to the
// heaviest, i.e. last, query block so that the last workgroups to start are the light ones).
__device__ __forceinline__ void map_workgroup(int L, int heads, int T_r, int head_group, int &head, int &qord) {
    if ((heads & 7) == 0) {
        const int s = L >> 3, per_group = head_group * T_r;
        const int grp = s / per_group, t = s % per_group;
        const int hpx = heads >> 3;                                  // heads per XCD
        const int gsz = min(head_group, hpx - grp * head_group);     // the last group may be short
        head = (grp * head_group + t % gsz) * 8 + (L & 7);
        qord = t / gsz;
    } else { head = L / T_r; qord = L % T_r; }
}

#if defined(__HIP_DEVICE_COMPILE__)   // buffer resources and LDS builtins do not exist in the host pass
struct BufRsrc { int w[4]; };        // raw buffer resource: base, base hi (stride 0), bytes, flags
__device__ __forceinline__ BufRsrc make_rsrc(const void *base, unsigned bytes) {
    const unsigned long long a = reinterpret_cast<unsigned long long>(base);
    BufRsrc r;                       // wave-uniform by construction; readfirstlane pins the words to SGPRs
    r.w[0] = __builtin_amdgcn_readfirstlane(static_cast<int>(static_cast<unsigned>(a)));
    r.w[1] = __builtin_amdgcn_readfirstlane(static_cast<int>(static_cast<unsigned>(a >> 32) & 0xffffu));
    r.w[2] = __builtin_amdgcn_readfirstlane(static_cast<int>(bytes));
    r.w[3] = 0x00020000;             // raw, 32-bit data format
    return r;
}

#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
// 64 lanes x 16 bytes: lane t's bytes [voff, voff + 16) past soff land at LDS address lds + 16 t
__device__ __forceinline__ void lds_copy16(const BufRsrc &r, lds_ptr lds, unsigned voff, int soff) {
    const v4i rs = {r.w[0], r.w[1], r.w[2], r.w[3]};
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :: "s"(static_cast<unsigned>(reinterpret_cast<uintptr_t>(lds))), "v"(voff), "s"(rs), "s"(soff) : "m0");
}
// the same with the non-temporal hint: for bytes that are read exactly once (the streaming passes of the key-split path)
__device__ __forceinline__ void lds_copy16_nt(const BufRsrc &r, lds_ptr lds, unsigned voff, int soff) {
    const v4i rs = {r.w[0], r.w[1], r.w[2], r.w[3]};
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, %3 offen nt lds"
                 :: "s"(static_cast<unsigned>(reinterpret_cast<uintptr_t>(lds))), "v"(voff), "s"(rs), "s"(soff) : "m0");
}
// 64 lanes x 4 bytes, lane t's dword lands at lds + 4 t
__device__ __forceinline__ void lds_copy4(const BufRsrc &r, lds_ptr lds, unsigned voff, int soff) {
    const v4i rs = {r.w[0], r.w[1], r.w[2], r.w[3]};
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dword %1, %2, %3 offen lds"
                 :: "s"(static_cast<unsigned>(reinterpret_cast<uintptr_t>(lds))), "v"(voff), "s"(rs), "s"(soff) : "m0");
}
#pragma clang diagnostic pop

// LDS address of an MFMA operand: (tile base + step) ^ lane offset.  Tile bases are multiples of 4096 and the lane
// offsets are below 4096, so the XOR that selects the step also adds the base: one vector instruction per address,
// the tile base and the step combined on the scalar side.
__device__ __forceinline__ lds_ptr lds_xor(lds_ptr base, unsigned step, unsigned lane_off) {
    const unsigned a = (static_cast<unsigned>(reinterpret_cast<uintptr_t>(base)) + step) ^ lane_off;
    return reinterpret_cast<lds_ptr>(static_cast<uintptr_t>(a));
}

// every outstanding memory operation of this wavefront has completed (vmcnt = expcnt = lgkmcnt = 0)
__device__ __forceinline__ void wait_all_memory() { __builtin_amdgcn_s_waitcnt(0); }

// a value that is the same in every lane, moved to a scalar register
__device__ __forceinline__ float uniform(float x) {
    return __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(x)));
}

// First MFMA of an accumulation chain: D = A B + ACC_START_I in every element, the constant being the instruction's
// inline operand 1 / (2 pi).  Written as assembly because the compiler folds a constant accumulator into the
// instruction only when that constant has a single use; otherwise it parks it in 16 registers.  The result is only
// ever read by the next MFMA of the chain (same registers as its accumulator, which may follow back to back).
__device__ __forceinline__ v16i mfma_i8_start(const v4i &a, const v4i &b) {
    v16i d;
    asm volatile("v_mfma_i32_32x32x32_i8 %0, %1, %2, 0.15915494" : "=&v"(d) : "v"(a), "v"(b));
    return d;
}

// Four P values, given as P / 65535, rounded to nearest and packed into the four bytes of a dword (key order):
// v_cvt_pknorm_u16_f32 twice (P in bytes 0 and 2 of each result), one v_perm_b32.
__device__ __forceinline__ uint32_t pack_p4(const float (&x)[4]) {
    typedef unsigned short us2 __attribute__((ext_vector_type(2)));
    const us2 lo = __builtin_amdgcn_cvt_pknorm_u16(x[0], x[1]), hi = __builtin_amdgcn_cvt_pknorm_u16(x[2], x[3]);
    return __builtin_amdgcn_perm(__builtin_bit_cast(uint32_t, hi), __builtin_bit_cast(uint32_t, lo), 0x06040200u);
}

// max (min) over the lane pair (r, r + 32) with v_permlane32_swap: no LDS round trip
__device__ __forceinline__ float pair_max(float x) {
    const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
}

__device__ __forceinline__ float pair_min(float x) {
    const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fminf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
}

#endif  // __HIP_DEVICE_COMPILE__

__device__ __forceinline__ float swap32(float x) {   // value held by lane ^ 32
    return __shfl_xor(x, 32);
}

// ---- output conversion --------------------------------------------------------------------------
// O is written once and never read back by these kernels: the whole-row stores of store_tile_staged carry the
// non-temporal hint, so that the output does not displace K and V in the L2 (+1.5 % on the headline workload).
// (Per-lane 8- and 16-byte pieces stored straight from the accumulator layout measured 2-6 % slower with the hint
// than without, and slower than the staged rows either way.)
template <typename T> struct Pack4;                 // four fp32 values -> four 2-byte outputs, round half to even
template <> struct Pack4<__half> {
    static __device__ __forceinline__ uint2 pack(float a, float b, float c, float d) {
        __half2 lo = __floats2half2_rn(a, b), hi = __floats2half2_rn(c, d);
        uint2 w;
        w.x = *reinterpret_cast<uint32_t *>(&lo);
        w.y = *reinterpret_cast<uint32_t *>(&hi);
        return w;
    }
};
template <> struct Pack4<__hip_bfloat16> {
    static __device__ __forceinline__ uint32_t rne(float x) {   // fp32 -> bf16 bits, round half to even; NaN stays NaN
        uint32_t u = __float_as_uint(x);
        return (x != x) ? 0x7fc0u : (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
    }
    static __device__ __forceinline__ uint2 pack(float a, float b, float c, float d) {
        uint2 w;
        w.x = rne(a) | (rne(b) << 16);
        w.y = rne(c) | (rne(d) << 16);
        return w;
    }
};

#if defined(__HIP_DEVICE_COMPILE__)
// Writes a wavefront's 32 x D output tile through a private LDS region of 64 D bytes so that the global stores are
// whole rows (2-byte outputs) or half rows (4-byte outputs, two passes over the region): in the accumulator layout a
// lane holds 4 consecutive d of one row per register group, and storing those directly costs one 8- or 16-byte
// piece per row and instruction.  Staged, lane t stores 16 contiguous bytes and 16 (D = 128) or 8 (D = 64) lanes
// cover a row piece of 2 D bytes.  The 16-byte chunks of a row are XOR-swizzled by the row so that the column-wise
// writes spread over the banks.  Only this wavefront touches `stage`; LDS operations of one wavefront complete in
// order, so no barrier is needed between the writes and the reads, or between the passes.
//   val(dt, v): element d = 32*dt + 8*(v/4) + 4*g + v%4 of row r = lane % 32 (g = lane / 32), already scaled
//   rows_valid: rows at or beyond it are not stored;  orow0: address of row 0 of the tile, row stride D elements
template <int D, typename OutT, typename F>
__device__ __forceinline__ void store_tile_staged(lds_ptr stage, OutT *orow0, int rows_valid, int lane, F val) {
    static_assert(sizeof(OutT) == 2 || sizeof(OutT) == 4, "2- or 4-byte outputs");
    constexpr int PASSES = sizeof(OutT) / 2;       // D/PASSES elements of every row per pass = 2 D bytes
    constexpr int DTP = (D / 32) / PASSES;         // 32-wide d tiles per pass
    constexpr int CH = D * 2 / 16;                 // 16-byte chunks per staged row piece
    constexpr int ROWS_PER_READ = 64 / CH;
    const int r = lane & 31, g = lane >> 5;
    const int c = lane % CH, rr = lane / CH;
#pragma unroll
    for (int pass = 0; pass < PASSES; ++pass) {
#pragma unroll
        for (int dl = 0; dl < DTP; ++dl)
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                const int dt = pass * DTP + dl;
                if constexpr (sizeof(OutT) == 2) {
                    const uint2 w = Pack4<OutT>::pack(val(dt, 4 * vq), val(dt, 4 * vq + 1), val(dt, 4 * vq + 2), val(dt, 4 * vq + 3));
                    *reinterpret_cast<LDS_AS uint2 *>(stage + r * (2 * D) + (((4 * dl + vq) ^ (r & (CH - 1))) * 16) + 8 * g) = w;
                } else {
                    const v4f w = {val(dt, 4 * vq), val(dt, 4 * vq + 1), val(dt, 4 * vq + 2), val(dt, 4 * vq + 3)};
                    *reinterpret_cast<LDS_AS v4f *>(stage + r * (2 * D) + (((8 * dl + 2 * vq + g) ^ (r & (CH - 1))) * 16)) = w;
                }
            }
#pragma unroll
        for (int rd = 0; rd < 32 / ROWS_PER_READ; ++rd) {
            const int row = rd * ROWS_PER_READ + rr;
            const v4i x = *reinterpret_cast<LDS_AS const v4i *>(stage + row * (2 * D) + ((c ^ (row & (CH - 1))) * 16));
            char *dst = reinterpret_cast<char *>(orow0 + static_cast<long>(row) * D) + pass * (2 * D) + 16 * c;
            if (row < rows_valid) __builtin_nontemporal_store(x, reinterpret_cast<v4i *>(dst));
        }
    }
}
#endif


}  // namespace ifa_dev

#endif  // INTFA_DEVICE_H
