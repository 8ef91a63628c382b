// Half-INT8 variant of the INT-FlashAttention forward pass for gfx950 (Section 4 of arXiv 2409.16997: INT8 Q and K
// with token-level scales, V kept in FP16).  The first GEMM and everything up to the running max are those of
// Algorithm 1; the softmax weights then stay real, are rounded to FP16 and meet the caller's FP16 V on
// v_mfma_f32_32x32x16_f16:
//     S^T = K_j Q_i^T                 v_mfma_i32_32x32x32_i8, fp32 scales             (lines 9-10)
//     P~  = fp16(exp(S - m))          no factor R; round to nearest even, subnormals kept
//     l   = alpha l + rowsum(P~)      the rounded weights, summed in fp32 (v_dot2_f32_f16 with ones)
//     O^T = alpha O^T + V_j^T P~^T    the MFMA accumulates straight onto the rescaled fp32 output
//     O   = O / l
//
// Same orientation and work split as the INT8 kernel (workgroup = 4 wavefronts = 128 queries, a lane owns one
// query), but the key block is B_c = 64: an FP16 V tile is twice the bytes of an INT8 one, and 64 keys keep
// K (2 x 8 KB) + V (2 x 16 KB) double-buffered at two workgroups per CU.  In the 32x32 accumulator layout a lane
// holds keys 8*(v/4) + 4*g + v%4 of a 32-key tile; two consecutive v/4 groups are the 8 contraction halves one
// lane feeds to a 32x32x16 MFMA, so P~ never leaves registers here either.  The matching V^T operand (8 keys of
// one d column per lane, V being [keys, d]) is gathered by the LDS with ds_read_b64_tr_b16: within 16 lanes,
// lane 4k+j addresses 4 halves (d = d0+4j .. +3) of key k, and lane i receives d column d0+i of keys 0..3.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <hip/hip_bf16.h>
#include <stdint.h>
#include <type_traits>

#include "intfa.h"
#include "intfa_internal.h"
#include "intfa_device.h"

namespace {

using namespace ifa_dev;

typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef short s4 __attribute__((ext_vector_type(4)));

constexpr int BCH = 64;       // keys per block of this variant
[[maybe_unused]] constexpr int NT = BCH / 32;  // 32-key tiles per block

template <int D> struct SmemH {
    alignas(4096) int8_t k[2][BCH * D];        // K_j int8, row = key, 16-byte slots XOR-swizzled by row
    alignas(1024) int8_t v[2][BCH * D * 2];    // V_j fp16, row = key (2 D bytes), 64-byte chunks XOR-swizzled by row
    alignas(256) float sk[2][BCH];             // s_K of the block
};
// lds_xor() wants every K / V tile at a multiple of 4096 bytes
static_assert((BCH * 64) % 4096 == 0 && offsetof(SmemH<64>, v) % 4096 == 0 && offsetof(SmemH<128>, v) % 4096 == 0, "tile bases");

template <int D> __device__ __forceinline__ int kh_swz(int row) {
    return (D == 128) ? (row & 7) : ((row >> 1) & 3);
}
// V rows are read 4 consecutive keys at a time at one 64-byte chunk: the low key bits pick the chunk slot
template <int D> __device__ __forceinline__ int vh_swz(int row) {
    return (D == 128) ? (row & 3) : (row & 1);
}

#if defined(__HIP_DEVICE_COMPILE__)

template <int D> struct LaneOffsetsH {
    static constexpr int KS = D / 32, DT = D / 32, KP = D / 64, VP = D / 32;
    // A operand of S^T: row r, 16-byte chunk 2*kk + g.  The swizzle XORs the chunk index and 2*kk + g = 2*kk ^ g,
    // so step kk is at k0 ^ (32*kk)   (+ 32*mt*D per key tile, an immediate)
    unsigned k0;
    // A operand of O^T: keys 4g + (i/4) of a 16-key step, d tile dt at v0 ^ (64*dt); the keys 8 further on, which the
    // swizzle does not see, at + 8 * 2D   (+ (32*mt + 16*s) * 2D per step)
    unsigned v0;
    // staging: byte offset inside the K / V block in HBM of the chunk this lane moves in piece 0 of its wavefront;
    // piece i is 1024 bytes further on (whole rows, which the swizzles do not see)
    unsigned gk, gv;
    __device__ __forceinline__ LaneOffsetsH(int lane, int wave) {
        const int r = lane & 31, g = lane >> 5;
        constexpr int CH = D / 16, CHV = D / 8;      // 16-byte slots per K row / per V row
        {
            const int p = wave * KP * 64 + lane, row = p / CH, slot = p % CH;      // a piece is 1024 / D >= 8 rows
            gk = row * D + 16 * (slot ^ kh_swz<D>(row));
        }
        {
            const int p = wave * VP * 64 + lane, row = p / CHV, slot = p % CHV;    // a piece is 512 / D >= 4 rows
            gv = row * (2 * D) + 16 * (slot ^ (vh_swz<D>(row) << 2));
        }
        k0 = r * D + ((g ^ kh_swz<D>(r)) * 16);
        const int i = lane & 15, G = lane >> 4, kq = i >> 2, j = i & 3;
        const int key = 4 * g + kq;
        v0 = key * (2 * D) + (vh_swz<D>(key) * 64) + 32 * (G & 1) + 8 * j;
    }
};

struct PrefetchH {
    BufRsrc k, v, sk;                // one head's K [N, d] int8, V [N, d] fp16 and s_K [N] fp32
    int koff, voff, skoff;           // byte offsets of the next block inside K, V and s_K
    lds_ptr lk, lv, lsk;             // LDS destinations
};
// Block offset of a request that must fetch nothing (no block follows): past the end of any tensor, so every lane
// is out of range (the scalar offset takes part in the range check) and the copy moves no data.
constexpr int NOWHERE_H = 0x7fff0000;

template <int D>
__device__ __forceinline__ void prefetch_block(const PrefetchH &nx, const LaneOffsetsH<D> &lo, int wave, int lane) {
    constexpr int KP = D / 64, VP = D / 32;
#pragma unroll
    for (int i = 0; i < KP; ++i) lds_copy16(nx.k, nx.lk + (wave * KP + i) * 1024, lo.gk, nx.koff + 1024 * i);
#pragma unroll
    for (int i = 0; i < VP; ++i) lds_copy16(nx.v, nx.lv + (wave * VP + i) * 1024, lo.gv, nx.voff + 1024 * i);
    if (wave == 3) lds_copy4(nx.sk, nx.lsk, 4 * lane, nx.skoff);       // 64 lanes x 4 bytes = the 64 scales of the block
}

template <int D> struct RowStateH {
    float m2;             // running max in log2 units (identical in lanes r and r + 32)
    float l;              // running sum of the rounded weights over this lane's keys
    v16f o[D / 32];       // running output, d = 32*dt + 8*(v/4) + 4*g + v%4: the MFMA accumulator itself
};

// One key block already resident in LDS.  MASKED: a block with masked keys (on or past the causal diagonal, or the
// ragged last block): a key of the block is kept iff its index inside the block is <= klimit (per lane, may be
// negative); the first `clear_tiles` 32-key tiles (wave-uniform) hold no masked key for any lane of the wavefront;
// 32-key tiles after tile `last` (wave-uniform, -1: none) are masked for every lane and skipped.
template <int D, bool MASKED>
__device__ __forceinline__ void process_block_half(lds_ptr ks, lds_ptr vs, lds_ptr sk, const LaneOffsetsH<D> &lo,
                                                   const v4i (&qf)[D / 32], float sq2, int klimit, int last_tile, int clear_tiles, int g,
                                                   const v16i &bias, RowStateH<D> &st) {
    constexpr int KS = D / 32, DT = D / 32;
    const int last = MASKED ? last_tile : NT - 1;
    float a[NT][16];
    float bmax = -INFINITY;

    // The source is software-pipelined like the INT8 kernel's: LDS operands of the next MFMA group are requested
    // before the current group is issued, and the vector work on tile t-1 follows the MFMAs of tile t.
    v4i kop[2][KS];
    v4f skr[2][4];
    auto load_k = [&](int buf, int mt) {
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) kop[buf][kk] = *reinterpret_cast<LDS_AS const v4i *>(lds_xor(ks, 32 * kk, lo.k0) + 32 * mt * D);
    };
    auto load_sk = [&](int buf, int mt) {
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) skr[buf][vq] = *reinterpret_cast<LDS_AS const v4f *>(sk + 16 * g + 128 * mt + 32 * vq);
    };
    auto scale_elems = [&](int mt, const v16i &acc, const v4f (&skv)[4], auto masked) {   // line 9, fp32 part: a = acc * s_K
#pragma unroll
        for (int vq = 0; vq < 4; ++vq)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float x = (__int_as_float(acc[4 * vq + e]) - ACC_BIAS_F) * skv[vq][e];
                if (decltype(masked)::value && (32 * mt + 8 * vq + 4 * g + e > klimit)) x = -INFINITY;   // masked key
                a[mt][4 * vq + e] = x;
                bmax = fmaxf(bmax, x);
            }
    };
    // only the tiles the mask boundary crosses pay for the comparisons (wave-uniform choice)
    auto scale_tile = [&](int mt, const v16i &acc, const v4f (&skv)[4]) {
        if (MASKED && mt >= clear_tiles) scale_elems(mt, acc, skv, std::true_type{});
        else scale_elems(mt, acc, skv, std::false_type{});
    };
    // V^T operands of d tile dt: one h8 per 16-key step of the active tiles
    h8 vop[2][2 * NT];
    auto load_v = [&](int buf, int dt) {
#pragma unroll
        for (int mt = 0; mt < NT; ++mt)
            if (mt <= last) {
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    const int koff = (32 * mt + 16 * s) * (2 * D);
                    const h4 t0 = __builtin_bit_cast(h4, __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<LDS_AS s4 *>(lds_xor(vs, 64 * dt, lo.v0) + koff)));
                    const h4 t1 = __builtin_bit_cast(h4, __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<LDS_AS s4 *>(lds_xor(vs, 64 * dt, lo.v0) + 8 * (2 * D) + koff)));
                    vop[buf][2 * mt + s] = h8{t0[0], t0[1], t0[2], t0[3], t1[0], t1[1], t1[2], t1[3]};
                }
            }
    };

    // ---- S^T = K Q^T, tile by tile
    v16i sacc[2];
    load_k(0, 0);
    load_sk(0, 0);
#pragma unroll
    for (int mt = 0; mt < NT; ++mt) {
        if (mt <= last) {
            if (mt + 1 <= last) load_k((mt + 1) & 1, mt + 1);
            sacc[mt & 1] = bias;
#pragma unroll
            for (int kk = 0; kk < KS; ++kk)
                sacc[mt & 1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(kop[mt & 1][kk], qf[kk], sacc[mt & 1], 0, 0, 0);
            if (mt > 0) scale_tile(mt - 1, sacc[(mt - 1) & 1], skr[(mt - 1) & 1]);
            if (mt + 1 <= last) load_sk((mt + 1) & 1, mt + 1);
        } else {
#pragma unroll
            for (int v = 0; v < 16; ++v) a[mt][v] = -INFINITY;
        }
    }
    if constexpr (MASKED) load_v(0, 0);                           // first V^T operands go out before the last tile is scaled
#pragma unroll
    for (int mt = 0; mt < NT; ++mt)
        if (mt == last) scale_tile(mt, sacc[mt & 1], skr[mt & 1]);

    bmax = pair_max(bmax);
    const float m_new = fmaxf(st.m2, bmax * sq2);                 // finite from the first block on (key 0 is never masked)
    const float alpha = __builtin_amdgcn_exp2f(st.m2 - m_new);    // exp2(-inf) = 0 on the first block
    st.m2 = m_new;

    // ---- P~ = fp16(2^(a s_Q' - m)), two keys per register in accumulator order; l sums the rounded values
    h2 ph[NT][8];
    float psum = 0.0f;
    const h2 ones = {(_Float16)1.0f, (_Float16)1.0f};
    auto p_pair = [&](int mt, int c) {
        const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(a[mt][2 * c], sq2, -m_new));
        const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(a[mt][2 * c + 1], sq2, -m_new));
        const h2 w = {(_Float16)p0, (_Float16)p1};
        ph[mt][c] = w;
        psum = __builtin_amdgcn_fdot2(w, ones, psum, false);
    };
    if constexpr (!MASKED) {
        // Unmasked blocks: the second GEMM runs key tile by key tile over all d tiles, with the weights of the NEXT key
        // tile computed between its MFMAs at raised wave priority (two exps per MFMA hide behind it); each V^T operand
        // is re-requested for the next key tile right after the MFMA that read it has issued.
        h8 vt[DT][2];
        auto load_v1 = [&](int mt, int dt, int s_) {
            const int koff = (32 * mt + 16 * s_) * (2 * D);
            const h4 t0 = __builtin_bit_cast(h4, __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<LDS_AS s4 *>(lds_xor(vs, 64 * dt, lo.v0) + koff)));
            const h4 t1 = __builtin_bit_cast(h4, __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<LDS_AS s4 *>(lds_xor(vs, 64 * dt, lo.v0) + 8 * (2 * D) + koff)));
            vt[dt][s_] = h8{t0[0], t0[1], t0[2], t0[3], t1[0], t1[1], t1[2], t1[3]};
        };
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) { load_v1(0, dt, 0); load_v1(0, dt, 1); }
#pragma unroll
        for (int c = 0; c < 8; ++c) p_pair(0, c);
        __builtin_amdgcn_s_setprio(3);
#pragma unroll
        for (int mt = 0; mt < NT; ++mt) {
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                if (mt == 0) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) st.o[dt][v] *= alpha;
                }
#pragma unroll
                for (int s_ = 0; s_ < 2; ++s_) {
                    const h8 pb = {ph[mt][4 * s_][0], ph[mt][4 * s_][1], ph[mt][4 * s_ + 1][0], ph[mt][4 * s_ + 1][1],
                                   ph[mt][4 * s_ + 2][0], ph[mt][4 * s_ + 2][1], ph[mt][4 * s_ + 3][0], ph[mt][4 * s_ + 3][1]};
                    st.o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vt[dt][s_], pb, st.o[dt], 0, 0, 0);
                    if (mt + 1 < NT) load_v1(mt + 1, dt, s_);
                }
                if (mt + 1 < NT) {
#pragma unroll
                    for (int q = 0; q < 8 / DT; ++q) p_pair(mt + 1, dt * (8 / DT) + q);
                }
            }
        }
        __builtin_amdgcn_s_setprio(0);
        st.l = __builtin_fmaf(st.l, alpha, psum);
        return;
    }
#pragma unroll
    for (int mt = 0; mt < NT; ++mt) {
        if (mt <= last) {
#pragma unroll
            for (int c = 0; c < 8; ++c) p_pair(mt, c);
        }
    }
    st.l = __builtin_fmaf(st.l, alpha, psum);

    // ---- O^T = alpha O^T + V^T P~^T: each d tile is rescaled in place, then the fp16 MFMAs accumulate onto it
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
        if (dt + 1 < DT) load_v((dt + 1) & 1, dt + 1);
#pragma unroll
        for (int v = 0; v < 16; ++v) st.o[dt][v] *= alpha;
#pragma unroll
        for (int mt = 0; mt < NT; ++mt) {
            if (mt <= last) {
#pragma unroll
                for (int s = 0; s < 2; ++s) {                       // 16-key steps of the tile
                    const h8 pb = {ph[mt][4 * s][0], ph[mt][4 * s][1], ph[mt][4 * s + 1][0], ph[mt][4 * s + 1][1],
                                   ph[mt][4 * s + 2][0], ph[mt][4 * s + 2][1], ph[mt][4 * s + 3][0], ph[mt][4 * s + 3][1]};
                    st.o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vop[dt & 1][2 * mt + s], pb, st.o[dt], 0, 0, 0);
                }
            }
        }
    }
}

#endif  // __HIP_DEVICE_COMPILE__

template <int D, bool CAUSAL, typename OutT>
__global__ __launch_bounds__(THREADS, 2) void int_flash_attn_fwd_half_kernel(
    const int8_t *__restrict__ Q, const int8_t *__restrict__ K, const _Float16 *__restrict__ V,
    const float *__restrict__ sQ, const float *__restrict__ sK, int heads, int Nq, int Nk, int head_group, OutT *__restrict__ O) {
#if defined(__HIP_DEVICE_COMPILE__)
    __shared__ SmemH<D> sm;
    constexpr int DT = D / 32;

    const int tid = threadIdx.x, lane = tid & 63, r = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int T_r = (Nq + BR - 1) / BR;
    const int T_c = (Nk + BCH - 1) / BCH;
    // Under the mask the queries are the LAST Nq positions of the key sequence: query i sees keys <= i + shift.
    const int shift = CAUSAL ? Nk - Nq : 0;

    int head, qord;
    map_workgroup(blockIdx.x, heads, T_r, head_group, head, qord);
    const int qb = CAUSAL ? (T_r - 1 - qord) : qord;
    const int q_local = 32 * wave + r;
    const int q_head = qb * BR + q_local;
    // rows past Nq are computed on a clamped copy of the last row and never stored
    const long qrow = static_cast<long>(head) * Nq + min(q_head, Nq - 1);

    const int8_t *Kh = K + static_cast<long>(head) * Nk * D;
    const _Float16 *Vh = V + static_cast<long>(head) * Nk * D;
    const float *sKh = sK + static_cast<long>(head) * Nk;
    const lds_ptr kbuf = (lds_ptr)(&sm.k[0][0]);
    const lds_ptr vbuf = (lds_ptr)(&sm.v[0][0]);
    const lds_ptr skbuf = (lds_ptr)(&sm.sk[0][0]);
    // key blocks this workgroup walks: up to the last key any of its queries sees
    const int first_q = qb * BR;
    const int nblocks = CAUSAL ? min(Nk - 1, first_q + BR - 1 + shift) / BCH + 1 : T_c;

    const BufRsrc rK = make_rsrc(Kh, static_cast<unsigned>(Nk) * D);
    const BufRsrc rV = make_rsrc(Vh, static_cast<unsigned>(Nk) * D * 2);
    const BufRsrc rSK = make_rsrc(sKh, static_cast<unsigned>(Nk) * 4);

    v4i qf[D / 32];
#pragma unroll
    for (int kk = 0; kk < D / 32; ++kk)
        qf[kk] = *reinterpret_cast<const v4i *>(Q + qrow * D + 32 * kk + 16 * g);
    const float sq2 = sQ[qrow] * LOG2E;
    const LaneOffsetsH<D> lo(lane, wave);
    {
        const PrefetchH first = {rK, rV, rSK, 0, 0, 0, kbuf, vbuf, skbuf};
        prefetch_block<D>(first, lo, wave, lane);
    }

    v16i bias;                                                   // constant registers the S^T accumulators start from
#pragma unroll
    for (int v = 0; v < 16; ++v) bias[v] = ACC_BIAS_I;
    asm volatile("" : "+v"(bias));                               // opaque: kept in registers, not re-materialised per use

    RowStateH<D> st;
    st.m2 = -INFINITY;
    st.l = 0.0f;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) st.o[dt][v] = 0.0f;

    wait_all_memory();
    __syncthreads();

    // Blocks in which every key counts for every query of the workgroup come first; the rest (the two blocks that
    // meet the causal diagonal band of the workgroup's 128 queries, or the ragged last block) run the masked code.
    const int nfull = min(nblocks, CAUSAL ? min(Nk / BCH, (first_q + shift + 1) / BCH) : Nk / BCH);
    const int wave_last_q = first_q + 32 * wave + 31;            // last query of this wavefront
    auto next_block = [&](int jb) {                              // what block jb + 1 needs staged, into the other buffers
        const int nxt = (jb & 1) ^ 1, j1 = (jb + 1) * BCH;
        const bool more = jb + 1 < nblocks;
        return PrefetchH{rK, rV, rSK, more ? j1 * D : NOWHERE_H, more ? j1 * D * 2 : NOWHERE_H, more ? j1 * 4 : NOWHERE_H,
                         kbuf + nxt * BCH * D, vbuf + nxt * BCH * D * 2, skbuf + nxt * BCH * 4};
    };
    for (int jb = 0; jb < nfull; ++jb) {
        const int cur = jb & 1;
        prefetch_block<D>(next_block(jb), lo, wave, lane);
        process_block_half<D, false>(kbuf + cur * BCH * D, vbuf + cur * BCH * D * 2, skbuf + cur * BCH * 4, lo, qf, sq2,
                                     0, NT - 1, NT, g, bias, st);
        wait_all_memory();                                       // my part of the next block has landed in LDS
        __syncthreads();                                         // everyone's has, and `cur` is free again
    }
    for (int jb = nfull; jb < nblocks; ++jb) {
        const int cur = jb & 1;
        prefetch_block<D>(next_block(jb), lo, wave, lane);
        const int j0 = jb * BCH;
        const int tail = Nk - 1 - j0;                                              // last valid key of the block
        const int klimit = CAUSAL ? min(q_head + shift - j0, tail) : tail;         // < 0: nothing kept
        const int wlim = CAUSAL ? min(wave_last_q + shift - j0, tail) : tail;
        const int last_tile = wlim < 0 ? -1 : min(NT - 1, wlim >> 5);
        const int wmin = CAUSAL ? min(wave_last_q - 31 + shift - j0, tail) : tail;   // klimit of the wavefront's first row
        if (last_tile >= 0)                                                        // wave-uniform
            process_block_half<D, true>(kbuf + cur * BCH * D, vbuf + cur * BCH * D * 2, skbuf + cur * BCH * 4, lo, qf, sq2,
                                        klimit, last_tile, max(0, (wmin + 1) >> 5), g, bias, st);
        wait_all_memory();
        __syncthreads();
    }

    const float l = st.l + swap32(st.l);
    const float f = 1.0f / l;
    // Every block ends with a barrier, so all of LDS is free here: each wavefront stages its 32 x D tile in its own
    // 64 D bytes of the V buffers and stores whole (fp32: half) rows.
    const int row0 = qb * BR + 32 * wave;                        // first query row of this wavefront
    OutT *orow0 = O + (static_cast<long>(head) * Nq + row0) * D;
    store_tile_staged<D, OutT>(vbuf + wave * (64 * D), orow0, Nq - row0, lane, [&](int dt, int v) { return st.o[dt][v] * f; });
#endif
}

template <int D, bool CAUSAL, typename OutT>
int launch_half(const int8_t *Q, const int8_t *K, const _Float16 *V, const float *sQ, const float *sK, int heads, int Nq, int Nk,
                void *O, hipStream_t st) {
    const long wgs = static_cast<long>(heads) * ((Nq + BR - 1) / BR);
    // T_r = 0: under the mask this kernel keeps 4 heads per group (8 measured 4-17 % slower here at N = 1280 .. 2048)
    hipLaunchKernelGGL((int_flash_attn_fwd_half_kernel<D, CAUSAL, OutT>), dim3(static_cast<unsigned>(wgs)), dim3(THREADS), 0,
                       st, Q, K, V, sQ, sK, heads, Nq, Nk, head_group_for(CAUSAL, 3L * Nk * D, 0), static_cast<OutT *>(O));
    return hipGetLastError() == hipSuccess ? IFA_OK : IFA_ERR_HIP;
}

template <int D, bool CAUSAL>
int launch_half_dtype(const int8_t *Q, const int8_t *K, const _Float16 *V, const float *sQ, const float *sK, int heads,
                      int Nq, int Nk, void *O, int o_dtype, hipStream_t st) {
    switch (o_dtype) {
    case IFA_F32: return launch_half<D, CAUSAL, float>(Q, K, V, sQ, sK, heads, Nq, Nk, O, st);
    case IFA_F16: return launch_half<D, CAUSAL, __half>(Q, K, V, sQ, sK, heads, Nq, Nk, O, st);
    default: return launch_half<D, CAUSAL, __hip_bfloat16>(Q, K, V, sQ, sK, heads, Nq, Nk, O, st);
    }
}

}  // namespace

extern "C" int ifa_block_cols_half(int d, int causal) {
    (void)causal;
    return (d == 64 || d == 128) ? BCH : 0;
}

namespace {
int half_entry(const signed char *Q_i8, const signed char *K_i8, const void *V_f16, const float *s_Q, const float *s_K,
               int B, int H, int Nq, int Nk, int d, int causal, void *O, int o_dtype, void *hip_stream) {
    if (!Q_i8 || !K_i8 || !V_f16 || !s_Q || !s_K || !O) return IFA_ERR_NULL;
    if (B <= 0 || H <= 0 || Nq <= 0 || Nk <= 0 || d <= 0) return IFA_ERR_SHAPE;
    const long heads = static_cast<long>(B) * H;
    const int N = Nq > Nk ? Nq : Nk;
    if (heads > (1L << 40) / N / d) return IFA_ERR_SHAPE;
    if (o_dtype < IFA_F32 || o_dtype > IFA_BF16) return IFA_ERR_DTYPE;
    if (d != 64 && d != 128) return IFA_ERR_UNSUPPORTED;
    if (causal && Nk < Nq) return IFA_ERR_UNSUPPORTED;           // a query with no visible key
    if (static_cast<long>(N) * d * 2 > 0x7ff00000L || heads * ((N + BR - 1) / BR) > 0x7fffffffL) return IFA_ERR_UNSUPPORTED;
    if (!ifa_aligned16(Q_i8) || !ifa_aligned16(K_i8) || !ifa_aligned16(V_f16) || !ifa_aligned16(O) ||
        (reinterpret_cast<uintptr_t>(s_Q) & 3) || (reinterpret_cast<uintptr_t>(s_K) & 3))
        return IFA_ERR_UNSUPPORTED;
    const int8_t *Q = reinterpret_cast<const int8_t *>(Q_i8);
    const int8_t *K = reinterpret_cast<const int8_t *>(K_i8);
    const _Float16 *V = reinterpret_cast<const _Float16 *>(V_f16);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const int hd = static_cast<int>(heads);
    if (d == 128)
        return causal ? launch_half_dtype<128, true>(Q, K, V, s_Q, s_K, hd, Nq, Nk, O, o_dtype, st)
                      : launch_half_dtype<128, false>(Q, K, V, s_Q, s_K, hd, Nq, Nk, O, o_dtype, st);
    return causal ? launch_half_dtype<64, true>(Q, K, V, s_Q, s_K, hd, Nq, Nk, O, o_dtype, st)
                  : launch_half_dtype<64, false>(Q, K, V, s_Q, s_K, hd, Nq, Nk, O, o_dtype, st);
}
}  // namespace

extern "C" int int_flash_attn_fwd_half(const signed char *Q_i8, const signed char *K_i8, const void *V_f16,
                                       const float *s_Q, const float *s_K, int B, int H, int N, int d, int causal,
                                       void *O, int o_dtype, void *hip_stream) {
    return half_entry(Q_i8, K_i8, V_f16, s_Q, s_K, B, H, N, N, d, causal, O, o_dtype, hip_stream);
}

extern "C" int int_flash_attn_fwd_half_rect(const signed char *Q_i8, const signed char *K_i8, const void *V_f16,
                                            const float *s_Q, const float *s_K, int B, int H, int Nq, int Nk, int d,
                                            int causal, void *O, int o_dtype, void *hip_stream) {
    return half_entry(Q_i8, K_i8, V_f16, s_Q, s_K, B, H, Nq, Nk, d, causal, O, o_dtype, hip_stream);
}
