// INT-FlashAttention forward (Algorithm 1) for gfx950: one fused kernel.
//
// Work split.  A workgroup of 4 wavefronts owns B_r = 128 query rows of one head, 32 per
// wavefront, and walks the key blocks of B_c = 128 keys in ascending order (Algorithm 1 lines
// 7-14).  K_j, V_j and s_K,j are copied HBM -> LDS with direct-to-LDS 128-bit loads
// (buffer_load_dwordx4 ... lds) into a double buffer, one block ahead of the arithmetic; everything
// else lives in registers.
//
// Orientation.  Both GEMMs are computed transposed on v_mfma_i32_32x32x32_i8:
//     S^T = K_j Q_i^T   (A = K_j rows from LDS, B = Q_i rows held in registers)
//     O^T = V_j^T P^T   (A = V_j^T rows from LDS, B = P^T, the packed softmax block)
// The 32x32 accumulator gives lane (c, g) = (lane % 32, lane / 32) column c and rows
// 8*(v/4) + 4*g + v%4, v = 0..15.  With queries as columns, a lane owns ONE query and 16 keys per
// 32-key tile: row max and row sum are in-lane plus one exchange with lane ^ 32, and the 16 P
// bytes a lane produces for a 32-key tile are exactly the 16 contraction bytes the B operand
// of the second GEMM wants from that lane -- P never leaves registers.  The contraction index of
// O^T = V^T P^T may be permuted freely as long as both operands agree, so the V^T operand is
// gathered with its keys in the order (tile, g, v) in which the accumulator layout delivers P.
//
// V_j is [keys, d] in HBM and LDS, and the MFMA wants 16 KEYS of one d column per lane: that byte
// transpose is done by the LDS itself with ds_read_b64_tr_b8 (per 16-lane group: lanes 0-7 receive
// byte column i of the 8 rows addressed by the even lanes, lanes 8-15 of the rows addressed by the
// odd lanes), two reads per MFMA operand, no VALU work.
//
// Softmax in base 2: log2(e) is folded into s_Q once per lane, the running max m2 is kept in log2 units and
// P = rint(127 exp2(acc * s_K * s_Q' - m2)) with one v_exp_f32 per score; the exponent also carries log2(127 / 65535),
// so that two v_cvt_pknorm_u16_f32 (round to nearest, measured) and one v_perm_b32 pack four P bytes into a dword.
//
// Schedule of one key block (the arrangement of this instruction mix that the issue-model micro-benchmark under
// csrc/microbench measured fastest on a gfx950 SIMD shared by two wavefronts):
//     M1  the 16 MFMAs of S^T back to back, into four accumulators that then become the scores in place
//     V1  scores: accumulator start taken off, times s_K, running extremum   (vector ALU only)
//     P0  P of the first 32-key tile: fma, exp2, pack                        (vector ALU + transcendental unit)
//     M2  the 16 MFMAs of O^T, key tile by key tile into four accumulators, with the P work of the NEXT key tile
//         between them, at raised wave priority: up to three v_exp_f32 fit under an MFMA of the same wavefront for free
//     --  wait for the staged copies, workgroup barrier, first K operands of the next block requested
//     V3  the four accumulators folded into the running output
// On this chip an MFMA and the plain vector instructions around it largely take turns instead of overlapping, whichever
// of the two wavefronts of the SIMD issues them (a wavefront that waits for the matrix pipe holds back its own vector
// stream behind it); only add, sub, mul and fma run at the full vector rate, everything else at half of it.
//
// The int32 results of both GEMMs are never converted: each accumulation chain starts from the MFMA's INLINE constant
// 1 / (2 pi) (bit pattern 0x3E22F983, in the middle of a binade where one integer step is 2^-26), so that a sum s reads
// as the float 1 / (2 pi) + s 2^-26, exactly, and one v_sub_f32 against the same inline constant recovers s 2^-26;
// no register holds the constant, and the 16 registers a constant block would take keep the query operands resident
// for the whole key loop.  Scores and the running output are carried in those units of 2^-26.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <hip/hip_bf16.h>
#include <stdint.h>
#include <type_traits>

#include "intfa.h"
#include "intfa_internal.h"
#include "intfa_attention_tiles.h"

// Wave priority inside the second GEMM (s_setprio; default priority elsewhere): measured best at 3 on long sequences.
#ifndef IFA_PRIO
#define IFA_PRIO 3
#endif

namespace {

using namespace ifa_tiles;

template <int D> struct Smem {
    alignas(4096) int8_t k[2][BC * D];   // K_j, row = key, 16-byte slots XOR-swizzled by row
    alignas(1024) int8_t v[2][BC * D];   // V_j, row = key, 16-byte slots XOR-swizzled by row
    alignas(512) float sk[2][BC];        // s_K of the block
};
// lds_xor() wants every K / V tile at a multiple of 4096 bytes
static_assert((BC * 64) % 4096 == 0 && offsetof(Smem<64>, v) % 4096 == 0 && offsetof(Smem<128>, v) % 4096 == 0, "tile bases");

// Test hook: where the int32 accumulators and the packed P of every key block go (null: not written), and an
// optional P to use in place of the computed one.  Only the DBG instantiation of the kernel reads this.
struct DebugDump {
    int *S;                // [Nq, Nk] int32: Q_i8 K_i8^T, the accumulator of line 9 minus its starting constant
    int8_t *P;             // [Nq, Nk] int8: P of line 11 as packed for the second GEMM
    int *PV;               // [T_c, Nq, d] int32: P_j V_j of line 13 per key block, accumulator minus its starting constant
    const int8_t *P_in;    // [Nq, Nk] int8 or null: replaces the computed P in the second GEMM (and in l)
    int Nk;
};

#if defined(__HIP_DEVICE_COMPILE__)   // device-only code: buffer resources and LDS builtins do not exist in the host pass
// ---- the fused kernel ---------------------------------------------------------------------------
// Online-softmax state of one lane: one query row, half of the keys of every block.
template <int D> struct RowState {
    float m2;             // running max in log2 units (identical in lanes r and r + 32)
    float l;              // running sum of the rounded P over this lane's keys
    float o[D / 32][16];  // the running output in units of 2^26, d = 32*dt + 8*(v/4) + 4*g + v%4
};

// Lines 9-13 of Algorithm 1 for one key block already resident in LDS.  DIAG: a block with masked keys --
// the block on the causal diagonal (query block == key block: keys beyond the query are masked) or the
// ragged last block (keys at or beyond N are masked).  A key of the block is kept iff its index inside the
// block is <= klimit (per lane); the first `clear_tiles` 32-key tiles (wave-uniform) hold no masked key for any
// lane of the wavefront; 32-key tiles after tile `last` (wave-uniform) are masked for every lane of
// the wavefront and are skipped (their P is 0).  `wave` is wave-uniform.
//
// !DIAG blocks also carry the block-to-block hand-over: they request the staging copies of the next block during
// M1, wait for them and meet the workgroup barrier between M2 and V3 (by then this wavefront has read everything
// it needs from the current buffers), and, if `preload_next`, request the first K operands of the next block right
// after the barrier so that their LDS latency is covered by V3.  `kfirst` holds those operands on entry and on
// exit.  DIAG blocks leave staging and barriers to the caller: a wavefront whose rows see none of a masked block
// skips it altogether.  In !DIAG blocks the issue order is pinned (sched_group_barrier) to the one written here.
template <int D, bool DIAG, bool VB, bool DBG>
__device__ __forceinline__ void process_block(lds_ptr ks, lds_ptr vs, lds_ptr sk, lds_ptr ks_next, const LaneOffsets<D> &lo,
                                              const v4i (&qf)[D / 32], float nq2, int wave, int lane, int klimit, int last_tile, int clear_tiles,
                                              int g, float oscale, const float *sv_next_ptr, float &sv_next, const Prefetch &nx, bool preload_next,
                                              v4i (&kfirst)[D / 32], RowState<D> &st, const DebugDump &dbg, long dbg_row, int dbg_j0, int dbg_jb, int dbg_nq) {
    constexpr int KS = D / 32, DT = D / 32;
    const int last = DIAG ? last_tile : 3;           // last active 32-key tile (wave-uniform)

    auto load_k = [&](v4i (&dst)[KS], lds_ptr base, int mt) {
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) dst[kk] = *reinterpret_cast<LDS_AS const v4i *>(k_operand<D>(base, lo, kk) + 32 * mt * D);
    };
    auto load_sk = [&](v4f (&dst)[4], int mt) {
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) dst[vq] = *reinterpret_cast<LDS_AS const v4f *>(sk + lo.sk + 128 * mt + 32 * vq);
    };

    // ---- M1: S^T = K Q^T, all four key tiles back to back (line 9, integer part).  The K operands of tile mt+1
    // are requested before the MFMAs of tile mt are issued; the staging copies of the next block go out here too.
    v16i sacc[4];
    v4i kop[2][KS];
    v4f skr[2][4];
    if (DIAG) load_k(kop[0], ks, 0);
    else {
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) kop[0][kk] = kfirst[kk];
    }
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
        if (mt <= last) {
            if (mt + 1 <= last) load_k(kop[(mt + 1) & 1], ks, mt + 1);
            // the scales of the first two key tiles are requested under the last MFMAs, so that V1 starts on data
            if (DIAG ? mt == last : mt == 2) load_sk(skr[0], 0);
            if (DIAG ? (mt == last && last >= 1) : mt == 3) load_sk(skr[1], 1);
            sacc[mt] = mfma_i8_start(kop[mt & 1][0], qf[0]);
#pragma unroll
            for (int kk = 1; kk < KS; ++kk)
                sacc[mt] = __builtin_amdgcn_mfma_i32_32x32x32_i8(kop[mt & 1][kk], qf[kk], sacc[mt], 0, 0, 0);
            if (!DIAG) {                                                    // issue order: operand reads, then this tile's MFMAs
                if (mt < 2) __builtin_amdgcn_sched_group_barrier(0x100, KS, 0);
                else if (mt == 2) __builtin_amdgcn_sched_group_barrier(0x100, KS + 4, 0);
                else __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, KS - 1, 0);     // (the chain start is an asm statement, not counted)
            }
            if (!DIAG && mt < KS) { prefetch_k_piece<D>(nx, lo, wave, mt); prefetch_v_piece<D>(nx, lo, wave, mt); }
        }
    }
    if (!DIAG) prefetch_sk(nx, wave, lane);
    __builtin_amdgcn_sched_barrier(0);

    if (DBG && dbg.S) {
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
            if (mt <= last)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int key = dbg_j0 + 32 * mt + 8 * (v >> 2) + 4 * g + (v & 3);
                    if (dbg_row < dbg_nq && key < dbg.Nk) dbg.S[dbg_row * dbg.Nk + key] = sacc[mt][v] - ACC_START_I;
                }
    }

    // ---- V1: line 9, fp32 part, in place of the accumulators.  t = ACC_START_F - acc = -(Q K^T) 2^-26 exactly, and
    // a = t * s_K: MINUS the score in units of 2^26 / (s_Q log2e); the per-row factor (negative: nq2) is applied after
    // the extremum, so the block maximum of line 10 is a minimum here and a masked key is +infinity.
    float a[4][16];
    float bmin = INFINITY;
    auto scale_elems = [&](int mt, const v4f (&skv)[4], auto masked) {
#pragma unroll
        for (int vq = 0; vq < 4; ++vq)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float x = (ACC_START_F - __int_as_float(sacc[mt][4 * vq + e])) * skv[vq][e];
                if (decltype(masked)::value && (32 * mt + 8 * vq + 4 * g + e > klimit)) x = INFINITY;   // masked key
                a[mt][4 * vq + e] = x;
                bmin = fminf(bmin, x);
            }
    };
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
        if (mt <= last) {
            // only the tiles the mask boundary crosses pay for the comparisons (wave-uniform choice)
            if (DIAG && mt >= clear_tiles) scale_elems(mt, skr[mt & 1], std::true_type{});
            else scale_elems(mt, skr[mt & 1], std::false_type{});
            if (mt + 2 <= last) load_sk(skr[mt & 1], mt + 2);    // into the registers this tile has just read
            if (!DIAG) {                                         // 16 subtractions, 16 multiplies, 8 three-way minima per tile
                __builtin_amdgcn_sched_group_barrier(0x002, 40, 0);
                if (mt < 2) __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
            }
        } else {
#pragma unroll
            for (int v = 0; v < 16; ++v) a[mt][v] = INFINITY;
        }
    }
    if (!DIAG) __builtin_amdgcn_sched_barrier(0);

    // line 10
    bmin = pair_min(bmin);
    const float m_new = fmaxf(st.m2, bmin * nq2);
    const float alpha = __builtin_amdgcn_exp2f(st.m2 - m_new);   // exp2(-inf) = 0 on the first block
    const float mm = m_new - LOG2_R_NORM;
    st.m2 = m_new;

    // line 11: P = rint(127 * 2^(a*s_Q' - m_new)), 4 keys per dword in accumulator order, one dword at a time.
    // The exponent carries log2(127 / 65535), so that the value is P / 65535 and the conversion to a 16-bit normalised
    // integer rounds it to P (to nearest; measured): two conversions give the four P of a dword in bytes 0 and 2 of two
    // registers, one byte permute gathers them -- three half-rate instructions where v_cvt_pk_u8_f32 takes four.
    v4i pf[4];
    uint32_t psum = 0;
    auto p_dword = [&](int mt, int vq) {
        float x[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) x[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(a[mt][4 * vq + e], nq2, -mm));
        uint32_t w = pack_p4(x);
        if (DBG && dbg.P_in) {
            const int key = dbg_j0 + 32 * mt + 8 * vq + 4 * g;
            w = (dbg_row < dbg_nq && key + 3 < dbg.Nk) ? *reinterpret_cast<const uint32_t *>(dbg.P_in + dbg_row * dbg.Nk + key) : 0u;
        }
        psum = __builtin_amdgcn_sad_u8(w, 0u, psum);
        pf[mt][vq] = static_cast<int>(w);
        if (DBG && dbg.P) {
            const int key = dbg_j0 + 32 * mt + 8 * vq + 4 * g;
            if (dbg_row < dbg_nq && key + 3 < dbg.Nk) *reinterpret_cast<uint32_t *>(dbg.P + dbg_row * dbg.Nk + key) = w;
        }
    };
    // ---- P0: the first key tile's P
#pragma unroll
    for (int vq = 0; vq < 4; ++vq) p_dword(0, vq);
    __builtin_amdgcn_sched_barrier(0);

    // ---- M2: line 13, O^T = V^T P^T key tile by key tile into DT accumulators; between the MFMAs of key tile mt
    // the P dwords of key tile mt + 1.  One V^T operand (two transposing reads) per MFMA, requested one key tile ahead
    // into the registers the previous MFMA of that d tile has read.
    v16i pacc[DT];
    v4i vop[DT];
    auto load_v = [&](int mt, int dt) {
        const v2i t0 = __builtin_amdgcn_ds_read_tr8_b64_v2i32(reinterpret_cast<LDS_AS v2i *>(v_operand<D>(vs, lo, dt) + 32 * mt * D));
        const v2i t1 = __builtin_amdgcn_ds_read_tr8_b64_v2i32(reinterpret_cast<LDS_AS v2i *>(v_operand<D>(vs, lo, dt) + 16 * D + 32 * mt * D));
        vop[dt] = v4i{t0[0], t0[1], t1[0], t1[1]};
    };
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) load_v(0, dt);
    if (IFA_PRIO) __builtin_amdgcn_s_setprio(IFA_PRIO);
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
        if (mt <= last) {
            if (!DIAG) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                pacc[dt] = mt == 0 ? mfma_i8_start(vop[dt], pf[0]) : __builtin_amdgcn_mfma_i32_32x32x32_i8(vop[dt], pf[mt], pacc[dt], 0, 0, 0);
                if (!DIAG && mt > 0) __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                if (mt + 1 <= last) {
                    load_v(mt + 1, dt);
                    if (!DIAG) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
#pragma unroll
                    for (int q = 0; q < 4 / DT; ++q) p_dword(mt + 1, dt * (4 / DT) + q);
                    if (!DIAG) {                                            // issue order: 4 fma, 4 exp2, 2 + 1 pack and the row sum per dword
                        __builtin_amdgcn_sched_group_barrier(0x002, 4 * (4 / DT), 0);
                        __builtin_amdgcn_sched_group_barrier(0x400, 4 * (4 / DT), 0);
                        __builtin_amdgcn_sched_group_barrier(0x002, 4 * (4 / DT), 0);
                    }
                }
            }
        }
    }
    if (!DIAG) __builtin_amdgcn_sched_barrier(0);
    if (IFA_PRIO) __builtin_amdgcn_s_setprio(0);
    if (DIAG) {
        // A wavefront that sees one key tile of a masked block ends every accumulation chain with its first MFMA, the
        // assembly statement the compiler does not know to be an MFMA: give those results time to land before the
        // fold reads them (everywhere else a chain ends with an MFMA of the compiler's own, which it waits for).
        asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15");
        __builtin_amdgcn_sched_barrier(0);
    }
    st.l = __builtin_fmaf(st.l, alpha, static_cast<float>(psum));   // line 12 (this lane's half of the keys)

    if (!DIAG) {
        // (VB) the next block's V scale: a scalar load placed where every counter is waited to zero anyway.  Anywhere
        // else, waiting for it means lgkmcnt(0), i.e. waiting for every LDS operand read in flight as well.
        if (VB) sv_next = *sv_next_ptr;
        wait_all_memory();                                       // my part of the next block has landed in LDS
        __syncthreads();                                         // everyone's has, and the current buffers are free again
        if (VB) asm volatile("" : "+s"(sv_next));
        if (preload_next) load_k(kfirst, ks_next, 0);
    }
    __builtin_amdgcn_sched_barrier(0);

    if (DBG && dbg.PV) {
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                if (dbg_row < dbg_nq)
                    dbg.PV[(static_cast<long>(dbg_jb) * dbg_nq + dbg_row) * D + 32 * dt + 8 * (v >> 2) + 4 * g + (v & 3)] = pacc[dt][v] - ACC_START_I;
    }

    // ---- V3: the running output is kept in units of 2^26: with t = ACC_START_F - acc = -(P V) 2^-26, exactly (one
    // v_sub_f32 with the inline constant), O' = alpha O - t is one fused multiply-add.  The negated addend needs the
    // three-address v_fma_f32, whose result can go back to O's own register; with a plain addend the compiler picks the
    // two-address v_fmac_f32, the result lands in t's register and every element costs a copy.
    // With one V scale per key block the running output is kept in units of the current block's scale:
    // O/s_j = (alpha s_{j-1}/s_j) (O/s_{j-1}) + P V_j, so the per-block scale costs one scalar multiply per lane.
    const float alpha_o = VB ? alpha * oscale : alpha;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v)
            st.o[dt][v] = __builtin_fmaf(st.o[dt][v], alpha_o, -(ACC_START_F - __int_as_float(pacc[dt][v])));
}

#endif  // __HIP_DEVICE_COMPILE__

template <int D, bool CAUSAL, bool VB, typename OutT, bool DBG = false>
__global__ __launch_bounds__(THREADS, 2) void int_flash_attn_fwd_kernel(
    const int8_t *__restrict__ Q, const int8_t *__restrict__ K, const int8_t *__restrict__ V,
    const float *__restrict__ sQ, const float *__restrict__ sK, const float *__restrict__ sV,
    int heads, int Nq, int Nk, int head_group, OutT *__restrict__ O, DebugDump dbg) {
#if defined(__HIP_DEVICE_COMPILE__)
    __shared__ Smem<D> sm;
    constexpr int DT = D / 32;

    const int tid = threadIdx.x, lane = tid & 63, r = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept in an SGPR
    const int T_r = (Nq + BR - 1) / BR;                          // the last query / key block may be ragged
    const int T_c = (Nk + BC - 1) / BC;
    // Under the mask the queries are the LAST Nq positions of the key sequence: query i sees keys <= i + shift.
    const int shift = CAUSAL ? Nk - Nq : 0;

    int head, qord;
    map_workgroup(blockIdx.x, heads, T_r, head_group, head, qord);
    const int qb = CAUSAL ? (T_r - 1 - qord) : qord;
    const int q_local = 32 * wave + r;                           // this lane's query inside the block
    const int q_head = qb * BR + q_local;                        // this lane's query inside the head
    // rows past Nq are computed on a clamped copy of the last row and never stored
    const long qrow = static_cast<long>(head) * Nq + min(q_head, Nq - 1);
    const long dbg_row = DBG ? q_head : 0;                       // the test hook runs one head

    const int8_t *Kh = K + static_cast<long>(head) * Nk * D;
    const int8_t *Vh = V + static_cast<long>(head) * Nk * D;
    const float *sKh = sK + static_cast<long>(head) * Nk;
    const lds_ptr kbuf = (lds_ptr)(&sm.k[0][0]);
    const lds_ptr vbuf = (lds_ptr)(&sm.v[0][0]);
    const lds_ptr skbuf = (lds_ptr)(&sm.sk[0][0]);
    // key blocks this workgroup walks: up to the last key any of its queries sees
    const int first_q = qb * BR;
    const int nblocks = CAUSAL ? min(Nk - 1, first_q + BR - 1 + shift) / BC + 1 : T_c;

    const BufRsrc rK = make_rsrc(Kh, static_cast<unsigned>(Nk) * D);
    const BufRsrc rV = make_rsrc(Vh, static_cast<unsigned>(Nk) * D);
    const BufRsrc rSK = make_rsrc(sKh, static_cast<unsigned>(Nk) * 4);

    // line 5: Q_i and s_Q,i.  B operand: lane (r, g) holds bytes d = 32*kk + 16*g .. +15 of query r.
    const int8_t *qptr = Q + qrow * D + 16 * g;
    v4i qf[D / 32];
#pragma unroll
    for (int kk = 0; kk < D / 32; ++kk) qf[kk] = *reinterpret_cast<const v4i *>(qptr + 32 * kk);
    const float nq2 = sQ[qrow] * (-LOG2E * ACC_UNIT);        // line 9's s_Q, log2 e, the accumulator unit and the sign of a
    const LaneOffsets<D> lo(lane, wave);
    {                                                            // line 8 for block 0
        const Prefetch first = {rK, rV, rSK, 0, 0, kbuf, vbuf, skbuf};
#pragma unroll
        for (int i = 0; i < D / 32; ++i) { prefetch_k_piece<D>(first, lo, wave, i); prefetch_v_piece<D>(first, lo, wave, i); }
        prefetch_sk(first, wave, lane);
    }

    // line 6
    RowState<D> st;
    st.m2 = -INFINITY;
    st.l = 0.0f;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) st.o[dt][v] = 0.0f;

    // Blocks in which every key counts for every query of the workgroup come first: all keys below Nk and, under
    // the mask, at or before the first query's last visible key.  The rest -- the block(s) the causal diagonal
    // crosses, the ragged last block -- run the masked code.
    const int nfull = min(nblocks, CAUSAL ? min(Nk / BC, (first_q + shift + 1) / BC) : Nk / BC);

    // s_V: one scalar per head, or (VB) one per key block of this head: sV [heads, T_c].  The scale of the coming block
    // is requested (a scalar load) in front of a wait for everything and handed on by the unmasked blocks: a scalar
    // load still in flight anywhere else turns every LDS wait behind it into a wait for all LDS reads.
    const float *sVh = VB ? sV + static_cast<long>(head) * T_c : sV + head;
    float sv_prev = 1.0f;
    float sv_cur = VB ? sVh[0] : 1.0f;
    wait_all_memory();
    __syncthreads();
    if (VB) asm volatile("" : "+s"(sv_cur));
    v4i kfirst[D / 32];                                          // K operands of the first key tile of the coming block
#pragma unroll
    for (int kk = 0; kk < D / 32; ++kk) kfirst[kk] = *reinterpret_cast<LDS_AS const v4i *>(k_operand<D>(kbuf, lo, kk));

    for (int jb = 0; jb < nfull; ++jb) {                         // line 7
        const int cur = jb & 1, nxt = cur ^ 1;
        const float sv_j = sv_cur;
        const float oscale = VB ? uniform(sv_prev * __builtin_amdgcn_rcpf(sv_j)) : 1.0f;
        sv_prev = sv_j;
        const int j1 = (jb + 1) * BC;                            // line 8 for the next block, asynchronous
        const bool more = jb + 1 < nblocks;
        const Prefetch pf = {rK, rV, rSK, more ? j1 * D : NOWHERE, more ? j1 * 4 : NOWHERE, kbuf + nxt * BC * D,
                             vbuf + nxt * BC * D, skbuf + nxt * BC * 4};
        // the staged copies are awaited and the workgroup barrier is met inside, between the second GEMM and the fold
        process_block<D, false, VB, DBG>(kbuf + cur * BC * D, vbuf + cur * BC * D, skbuf + cur * BC * 4, kbuf + nxt * BC * D, lo, qf, nq2,
                                         wave, lane, 0, 3, 4, g, oscale, sVh + (VB ? min(jb + 1, T_c - 1) : 0), sv_cur, pf, jb + 1 < nfull, kfirst, st, dbg,
                                         dbg_row, jb * BC, jb, Nq);
    }
    // At most two masked blocks follow (the diagonal band of 128 queries crosses at most two key blocks, and the
    // ragged last block is one of them or, without a mask, the only one).  They are written out one after the
    // other rather than as a loop so that the staging offsets are dead once the second one has been requested.
    auto masked_block = [&](int jb) {
        const int cur = jb & 1, j0 = jb * BC;
        // kept keys of this block: index inside the block <= klimit (may be negative: none).  Tiles after tile
        // wlim / 32 hold no kept key for any lane of this wavefront.
        const int tail = Nk - 1 - j0;
        const int klimit = CAUSAL ? min(q_head + shift - j0, tail) : tail;
        const int wlim = CAUSAL ? min(first_q + 32 * wave + 31 + shift - j0, tail) : tail;
        const int wmin = CAUSAL ? min(first_q + 32 * wave + shift - j0, tail) : tail;   // klimit of the wavefront's first row
        if (wlim >= 0) {                                         // wave-uniform: this wavefront sees part of the block
            const Prefetch none = {rK, rV, rSK, NOWHERE, NOWHERE, kbuf, vbuf, skbuf};   // masked blocks request nothing
            const float sv_j = VB ? (jb == nfull ? sv_cur : uniform(sVh[jb])) : 1.0f;
            const float oscale = VB ? uniform(sv_prev * __builtin_amdgcn_rcpf(sv_j)) : 1.0f;
            sv_prev = sv_j;
            process_block<D, true, VB, DBG>(kbuf + cur * BC * D, vbuf + cur * BC * D, skbuf + cur * BC * 4, kbuf, lo, qf, nq2, wave, lane,
                                            klimit, min(3, wlim >> 5), max(0, (wmin + 1) >> 5), g, oscale, sVh, sv_cur, none, false, kfirst, st, dbg,
                                            dbg_row, j0, jb, Nq);
        }
    };
    if (nfull < nblocks) {
        const bool second = nfull + 1 < nblocks;
        if (second) {                                            // line 8 for the second masked block
            const int nxt = (nfull & 1) ^ 1, j1 = (nfull + 1) * BC;
            const Prefetch pf = {rK, rV, rSK, j1 * D, j1 * 4, kbuf + nxt * BC * D, vbuf + nxt * BC * D, skbuf + nxt * BC * 4};
#pragma unroll
            for (int i = 0; i < D / 32; ++i) { prefetch_k_piece<D>(pf, lo, wave, i); prefetch_v_piece<D>(pf, lo, wave, i); }
            prefetch_sk(pf, wave, lane);
        }
        masked_block(nfull);
        if (second) {
            wait_all_memory();
            __syncthreads();
            masked_block(nfull + 1);
        }
    }

    // lines 15-17: O_i = diag(l)^-1 O s_V.  Lane (r, g) holds d = 32*dt + 8*(v/4) + 4*g + v%4.
    const float l = st.l + swap32(st.l);
    const float f = (VB ? sv_prev : sVh[0]) * ACC_UNIT / l;      // st.o holds O 2^-26 (in units of the last block's scale if VB)
    // The buffers the last block did not use are free for every wavefront since the barrier before it: each
    // wavefront stages its tile in its own 64 D bytes of them and stores whole (fp32: half) rows.
    const int freeb = nblocks & 1;
    const lds_ptr stage = (wave < 2 ? kbuf : vbuf) + freeb * BC * D + (wave & 1) * (64 * D);
    const int row0 = qb * BR + 32 * wave;                        // first query row of this wavefront
    OutT *orow0 = O + (static_cast<long>(head) * Nq + row0) * D;
    store_tile_staged<D, OutT>(stage, orow0, Nq - row0, lane, [&](int dt, int v) { return st.o[dt][v] * f; });
#endif
}

// ---- host side ----------------------------------------------------------------------------------
hipStream_t g_stream = nullptr;

template <int D, bool CAUSAL, bool VB, typename OutT>
int launch_fwd(const int8_t *Q, const int8_t *K, const int8_t *V, const float *sQ, const float *sK, const float *sV,
               int heads, int Nq, int Nk, void *O, hipStream_t st) {
    const long wgs = static_cast<long>(heads) * ((Nq + BR - 1) / BR);
    hipLaunchKernelGGL((int_flash_attn_fwd_kernel<D, CAUSAL, VB, OutT>), dim3(static_cast<unsigned>(wgs)), dim3(THREADS), 0,
                       st, Q, K, V, sQ, sK, sV, heads, Nq, Nk, head_group_for(CAUSAL, 2L * Nk * D, (Nq + BR - 1) / BR), static_cast<OutT *>(O),
                       DebugDump{nullptr, nullptr, nullptr, nullptr, 0});
    return hipGetLastError() == hipSuccess ? IFA_OK : IFA_ERR_HIP;
}

// Calls with at most this many queries per head go to the narrow kernel of intfa_attention_fewq.hip (measured against
// the fused kernel).
#ifndef IFA_NARROW_MAX_Q
#define IFA_NARROW_MAX_Q 64
#endif

template <int D, bool CAUSAL, bool VB>
int launch_fwd_dtype(const int8_t *Q, const int8_t *K, const int8_t *V, const float *sQ, const float *sK,
                     const float *sV, int heads, int Nq, int Nk, void *O, int o_dtype, hipStream_t st) {
    if (Nq <= IFA_NARROW_MAX_Q)
        return ifa_launch_narrow(Q, K, V, sQ, sK, sV, heads, Nq, Nk, D, CAUSAL ? 1 : 0, VB ? 1 : 0, O, o_dtype, st);
    switch (o_dtype) {
    case IFA_F32: return launch_fwd<D, CAUSAL, VB, float>(Q, K, V, sQ, sK, sV, heads, Nq, Nk, O, st);
    case IFA_F16: return launch_fwd<D, CAUSAL, VB, __half>(Q, K, V, sQ, sK, sV, heads, Nq, Nk, O, st);
    default: return launch_fwd<D, CAUSAL, VB, __hip_bfloat16>(Q, K, V, sQ, sK, sV, heads, Nq, Nk, O, st);
    }
}

// validation and dispatch shared by the tensor-level and the block-level V scale entry points
template <bool VB>
int fwd_entry(const signed char *Q_i8, const signed char *K_i8, const signed char *V_i8, const float *s_Q,
              const float *s_K, const float *s_V, int B, int H, int Nq, int Nk, int d, int causal, void *O, int o_dtype,
              void *hip_stream) {
    if (!Q_i8 || !K_i8 || !V_i8 || !s_Q || !s_K || !s_V || !O) return IFA_ERR_NULL;
    if (B <= 0 || H <= 0 || Nq <= 0 || Nk <= 0 || d <= 0) return IFA_ERR_SHAPE;
    const long heads = static_cast<long>(B) * H;
    const int N = Nq > Nk ? Nq : Nk;
    if (heads > (1L << 40) / N / d) return IFA_ERR_SHAPE;
    if (causal && Nk < Nq) return IFA_ERR_UNSUPPORTED;           // a query with no visible key
    if (o_dtype < IFA_F32 || o_dtype > IFA_BF16) return IFA_ERR_DTYPE;
    if (d != 64 && d != 128) return IFA_ERR_UNSUPPORTED;
    if (static_cast<long>(N) * d > 0x7ff00000L ||   // a head's K (or V) stays below NOWHERE
         heads * ((N + BR - 1) / BR) > 0x7fffffffL) return IFA_ERR_UNSUPPORTED;
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
        return causal ? launch_fwd_dtype<128, true, VB>(Q, K, V, s_Q, s_K, s_V, hd, Nq, Nk, O, o_dtype, st)
                      : launch_fwd_dtype<128, false, VB>(Q, K, V, s_Q, s_K, s_V, hd, Nq, Nk, O, o_dtype, st);
    return causal ? launch_fwd_dtype<64, true, VB>(Q, K, V, s_Q, s_K, s_V, hd, Nq, Nk, O, o_dtype, st)
                  : launch_fwd_dtype<64, false, VB>(Q, K, V, s_Q, s_K, s_V, hd, Nq, Nk, O, o_dtype, st);
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
    case IFA_ERR_WORKSPACE: return "IFA_ERR_WORKSPACE: the shape needs more workspace than was given (or than the static workspace holds)";
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
    return fwd_entry<false>(Q_i8, K_i8, V_i8, s_Q, s_K, s_V, B, H, N, N, d, causal, O, o_dtype, hip_stream);
}

extern "C" int int_flash_attn_fwd_vblock(const signed char *Q_i8, const signed char *K_i8, const signed char *V_i8,
                                         const float *s_Q, const float *s_K, const float *s_Vb, int B, int H, int N,
                                         int d, int causal, void *O, int o_dtype, void *hip_stream) {
    return fwd_entry<true>(Q_i8, K_i8, V_i8, s_Q, s_K, s_Vb, B, H, N, N, d, causal, O, o_dtype, hip_stream);
}

extern "C" int int_flash_attn_fwd_vblock_rect(const signed char *Q_i8, const signed char *K_i8, const signed char *V_i8,
                                              const float *s_Q, const float *s_K, const float *s_Vb, int B, int H, int Nq,
                                              int Nk, int d, int causal, void *O, int o_dtype, void *hip_stream) {
    return fwd_entry<true>(Q_i8, K_i8, V_i8, s_Q, s_K, s_Vb, B, H, Nq, Nk, d, causal, O, o_dtype, hip_stream);
}

extern "C" int int_flash_attn_fwd_rect(const signed char *Q_i8, const signed char *K_i8, const signed char *V_i8,
                                       const float *s_Q, const float *s_K, const float *s_V, int B, int H, int Nq, int Nk,
                                       int d, int causal, void *O, int o_dtype, void *hip_stream) {
    return fwd_entry<false>(Q_i8, K_i8, V_i8, s_Q, s_K, s_V, B, H, Nq, Nk, d, causal, O, o_dtype, hip_stream);
}

extern "C" int int_flash_attn_fwd(const signed char *Q_i8, const signed char *K_i8, const signed char *V_i8,
                                  const float *s_Q, const float *s_K, const float *s_V, int B, int H, int N, int d,
                                  int causal, void *O) {
    return int_flash_attn_fwd_ex(Q_i8, K_i8, V_i8, s_Q, s_K, s_V, B, H, N, d, causal, O, IFA_F16, g_stream);
}

// Test hook: the production kernel (the DBG instantiation differs only by the stores below the accumulators)
// on one head, with the integer stages written out.
template <int D, bool CAUSAL>
static int launch_debug(const int8_t *Q, const int8_t *K, const int8_t *V, const float *sQ, const float *sK, const float *sV, int N,
                 const DebugDump &dbg, float *O, hipStream_t st) {
    hipLaunchKernelGGL((int_flash_attn_fwd_kernel<D, CAUSAL, false, float, true>), dim3(N / BR), dim3(THREADS), 0, st, Q, K, V, sQ, sK,
                       sV, 1, N, N, 1, O, dbg);
    return hipGetLastError() == hipSuccess ? IFA_OK : IFA_ERR_HIP;
}

extern "C" int ifa_debug_fwd(const signed char *Q_i8, const signed char *K_i8, const signed char *V_i8, const float *s_Q,
                             const float *s_K, const float *s_V, int N, int d, int causal, const signed char *P_in, int *S_i32,
                             signed char *P_i8, int *PV_i32, float *O, void *hip_stream) {
    if (!Q_i8 || !K_i8 || !V_i8 || !s_Q || !s_K || !s_V || !O) return IFA_ERR_NULL;
    if (N <= 0 || d <= 0) return IFA_ERR_SHAPE;
    if ((d != 64 && d != 128) || N % BR != 0 || N > 8192) return IFA_ERR_UNSUPPORTED;
    if (!ifa_aligned16(Q_i8) || !ifa_aligned16(K_i8) || !ifa_aligned16(V_i8) || !ifa_aligned16(O) ||
        (reinterpret_cast<uintptr_t>(S_i32) & 3) || (reinterpret_cast<uintptr_t>(PV_i32) & 3) ||
        (reinterpret_cast<uintptr_t>(P_in) & 3) || (reinterpret_cast<uintptr_t>(P_i8) & 3) ||
        (reinterpret_cast<uintptr_t>(s_Q) & 3) || (reinterpret_cast<uintptr_t>(s_K) & 3) || (reinterpret_cast<uintptr_t>(s_V) & 3))
        return IFA_ERR_UNSUPPORTED;
    const int8_t *Q = reinterpret_cast<const int8_t *>(Q_i8);
    const int8_t *K = reinterpret_cast<const int8_t *>(K_i8);
    const int8_t *V = reinterpret_cast<const int8_t *>(V_i8);
    const DebugDump dbg = {S_i32, reinterpret_cast<int8_t *>(P_i8), PV_i32, reinterpret_cast<const int8_t *>(P_in), N};
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (d == 128)
        return causal ? launch_debug<128, true>(Q, K, V, s_Q, s_K, s_V, N, dbg, O, st) : launch_debug<128, false>(Q, K, V, s_Q, s_K, s_V, N, dbg, O, st);
    return causal ? launch_debug<64, true>(Q, K, V, s_Q, s_K, s_V, N, dbg, O, st) : launch_debug<64, false>(Q, K, V, s_Q, s_K, s_V, N, dbg, O, st);
}

