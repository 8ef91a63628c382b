// INT-FlashAttention forward (Algorithm 1) for gfx950: calls with few queries per head (a decode step, a few draft
// tokens, a short chunk of a prefill).  Two families, both built from the tile code of the fused kernel
// (intfa_attention_tiles.h: same LDS layout, same MFMA operand order, same staging copies) and the same arithmetic:
//   int_flash_attn_fwd_narrow_kernel   one workgroup per head and group of 32 queries, each key block split over its
//                                      four wavefronts; bit-identical to the fused kernel's rows, needs no memory
//                                      beyond inputs and outputs; what int_flash_attn_fwd_rect runs for N_q <= 64;
//   splitk_*                           the key axis of a head split over many workgroups, exactly: lines 9-10 for every
//                                      block first, then lines 11-13 on the known running maximum, then a merge;
//                                      int_flash_attn_fwd_splitk (caller's workspace) and _splitk_static (built in).
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <hip/hip_bf16.h>
#include <stdint.h>
#include <mutex>
#include <type_traits>

#include "intfa.h"
#include "intfa_internal.h"
#include "intfa_attention_tiles.h"

namespace {

using namespace ifa_tiles;

// ---- few queries, many keys (a decode step, a short chunk of a prefill) ---------------------------------------
// With at most a few dozen queries per head the fused kernel would keep three of its four wavefronts idle and one
// workgroup per head cannot fill the chip; what limits such a call is how fast K and V stream in.  Here the four
// wavefronts of a workgroup share ONE group of 32 queries and split each 128-key block instead:
//     wavefront w computes S^T for key tile w (32 keys; 4 MFMAs), scales it, takes its minimum / maximum;
//     the four per-query extrema meet in LDS (first barrier of the block): everyone knows m of line 10 for the whole block;
//     wavefront w computes the 16 P bytes per lane of its key tile and leaves them in LDS (second barrier);
//     wavefront w then computes the d tile w (32 of the d columns) of O^T = V^T P^T over ALL 128 keys (4 MFMAs,
//     P operands of the four key tiles from LDS) and folds it into its 16 registers of the running output.
// Every number is computed by the same instruction sequence on the same operands as in the fused kernel (the
// integer sums are exact, the extremum is order-independent, the row sum l is taken over the same P dwords), so
// the output is bit-identical to the corresponding rows of a square call: still Algorithm 1 at B_c = 128.
// K and V come in through a ring of NSTAGE blocks (one workgroup per CU: there are few workgroups anyway), filled
// three blocks ahead so that enough bytes are in flight to cover the HBM latency; the wait for a block is a
// counted s_waitcnt (every wavefront issues the same number of copy instructions per block) in front of the second
// barrier of the block before, which thereby also publishes the staged block; the first barrier releases the
// stage of the block before for refilling.
constexpr int NARROW_BR = 32;      // queries per workgroup
constexpr int NSTAGE = 4;

template <int D> struct SmemNarrow {
    alignas(4096) int8_t k[NSTAGE][BC * D];
    alignas(4096) int8_t v[NSTAGE][BC * D];
    alignas(512) float sk[NSTAGE][BC];
    alignas(16) float ext[4][32];          // per key tile and query: the tile's extremum of a (line 10)
    alignas(16) v4i p[4][64];              // per key tile and lane: the 16 P bytes of that lane (line 11)
};
static_assert(sizeof(SmemNarrow<128>) <= 160 * 1024 && offsetof(SmemNarrow<64>, v) % 4096 == 0, "LDS budget and tile bases");

template <int D, bool CAUSAL, bool VB, typename OutT>
__global__ __launch_bounds__(THREADS) void int_flash_attn_fwd_narrow_kernel(
    const int8_t *__restrict__ Q, const int8_t *__restrict__ K, const int8_t *__restrict__ V,
    const float *__restrict__ sQ, const float *__restrict__ sK, const float *__restrict__ sV,
    int heads, int Nq, int Nk, OutT *__restrict__ O) {
#if defined(__HIP_DEVICE_COMPILE__)
    __shared__ SmemNarrow<D> sm;
    constexpr int KS = D / 32;
    constexpr int PER_BLOCK = 2 * KS + 1;                        // copy instructions per wavefront and block

    const int tid = threadIdx.x, lane = tid & 63, r = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int T_c = (Nk + BC - 1) / BC;
    const int qgroups = (Nq + NARROW_BR - 1) / NARROW_BR;
    const int shift = CAUSAL ? Nk - Nq : 0;
    // all query groups of a head on one XCD (workgroups go round-robin over the 8 XCDs by linear id)
    int head, qg;
    if ((heads & 7) == 0) { const int s_ = blockIdx.x >> 3; head = (s_ / qgroups) * 8 + (blockIdx.x & 7); qg = s_ % qgroups; }
    else { head = blockIdx.x / qgroups; qg = blockIdx.x % qgroups; }
    const int first_q = qg * NARROW_BR;
    const int q_head = first_q + r;
    const long qrow = static_cast<long>(head) * Nq + min(q_head, Nq - 1);   // rows past Nq: a clamped copy, never stored

    const int8_t *Kh = K + static_cast<long>(head) * Nk * D;
    const int8_t *Vh = V + static_cast<long>(head) * Nk * D;
    const float *sKh = sK + static_cast<long>(head) * Nk;
    const lds_ptr kbuf = (lds_ptr)(&sm.k[0][0]);
    const lds_ptr vbuf = (lds_ptr)(&sm.v[0][0]);
    const lds_ptr skbuf = (lds_ptr)(&sm.sk[0][0]);
    const int nblocks = CAUSAL ? min(Nk - 1, min(first_q + NARROW_BR, Nq) - 1 + shift) / BC + 1 : T_c;

    const BufRsrc rK = make_rsrc(Kh, static_cast<unsigned>(Nk) * D);
    const BufRsrc rV = make_rsrc(Vh, static_cast<unsigned>(Nk) * D);
    const BufRsrc rSK = make_rsrc(sKh, static_cast<unsigned>(Nk) * 4);
    const LaneOffsets<D> lo(lane, wave);

    // line 8 for block jb into stage jb % NSTAGE; a block past the last one is requested nowhere (no data moves), so
    // that every block costs every wavefront PER_BLOCK copy instructions and the counted wait below stays valid
    auto stage_block = [&](int jb) {
        const int st = jb % NSTAGE;
        const bool real = jb < nblocks;
        const Prefetch pf = {rK, rV, rSK, real ? jb * BC * D : NOWHERE, real ? jb * BC * 4 : NOWHERE,
                             kbuf + st * BC * D, vbuf + st * BC * D, skbuf + st * BC * 4};
#pragma unroll
        for (int i = 0; i < KS; ++i) { prefetch_k_piece<D>(pf, lo, wave, i); prefetch_v_piece<D>(pf, lo, wave, i); }
        lds_copy4(pf.sk, pf.lsk + 256 * (wave & 1), 4 * lane + 256 * (wave & 1), pf.skoff);   // wavefronts 2, 3 repeat 0, 1
    };
    stage_block(0);
    stage_block(1);
    stage_block(2);

    // line 5
    const int8_t *qptr = Q + qrow * D + 16 * g;
    v4i qf[KS];
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) qf[kk] = *reinterpret_cast<const v4i *>(qptr + 32 * kk);
    float nq2 = sQ[qrow] * (-LOG2E * ACC_UNIT);
    // The loads above must have landed BEFORE the loop as far as the compiler is concerned: a wait for them inside the
    // loop would be a wait for every outstanding vector-memory operation, the staged copies included.
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) asm volatile("" : "+v"(qf[kk]));
    asm volatile("" : "+v"(nq2));

    // line 6: this wavefront's d tile of the running output (units of 2^26), m and l of the whole row
    float m2 = -INFINITY, l = 0.0f, o[16];
    v16i acc0;                                                   // what both accumulations start from
#pragma unroll
    for (int v = 0; v < 16; ++v) { o[v] = 0.0f; acc0[v] = ACC_START_I; }

    // s_V: one scalar per head, or (VB) one per key block of this head, read through the scalar cache
    const float *sVh = VB ? sV + static_cast<long>(head) * T_c : sV + head;
    float sv_prev = 1.0f;
    wait_vmcnt<2 * PER_BLOCK>();                                 // my pieces of block 0 have landed (blocks 1 and 2 may be in flight)
    __syncthreads();                                             // everyone's have
    for (int jb = 0; jb < nblocks; ++jb) {                       // line 7
        const int st = jb % NSTAGE, j0 = jb * BC;
        // with one V scale per key block the running output is kept in units of the current block's scale (as in the fused kernel)
        const float sv_j = VB ? uniform(sVh[jb]) : 1.0f;
        const float oscale = VB ? uniform(sv_prev * __builtin_amdgcn_rcpf(sv_j)) : 1.0f;
        sv_prev = sv_j;
        const lds_ptr ks = kbuf + st * BC * D, vs = vbuf + st * BC * D, sk = skbuf + st * BC * 4;

        // line 9 for key tile `wave`
        v4i kop[KS];
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) kop[kk] = *reinterpret_cast<LDS_AS const v4i *>(k_operand<D>(ks, lo, kk) + 32 * wave * D);
        v4f skv[4];
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) skv[vq] = *reinterpret_cast<LDS_AS const v4f *>(sk + lo.sk + 128 * wave + 32 * vq);
        // (registers are plentiful here: the accumulators start from a register block holding the constant, and every
        // MFMA is the compiler's own, with its dependency handling)
        v16i sacc = acc0;
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) sacc = __builtin_amdgcn_mfma_i32_32x32x32_i8(kop[kk], qf[kk], sacc, 0, 0, 0);
        // kept keys: index inside the block <= klimit (the causal diagonal, the ragged end of the sequence)
        const int tail = Nk - 1 - j0;
        const int klimit = CAUSAL ? min(q_head + shift - j0, tail) : tail;
        const bool masked = CAUSAL ? (j0 + BC - 1 > min(first_q + shift, Nk - 1)) : (tail < BC - 1);   // wave-uniform
        float a[16], bmin = INFINITY;
#pragma unroll
        for (int vq = 0; vq < 4; ++vq)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float x = (ACC_START_F - __int_as_float(sacc[4 * vq + e])) * skv[vq][e];
                if (masked && (32 * wave + 8 * vq + 4 * g + e > klimit)) x = INFINITY;
                a[4 * vq + e] = x;
                bmin = fminf(bmin, x);
            }
        bmin = pair_min(bmin);
        if (g == 0) sm.ext[wave][r] = bmin;
        __syncthreads();
        // every wavefront is past the second GEMM of block jb - 1: the stage that block used takes block jb + 3
        stage_block(jb + 3);
        // line 10 over the whole block
        bmin = fminf(fminf(sm.ext[0][r], sm.ext[1][r]), fminf(sm.ext[2][r], sm.ext[3][r]));
        const float m_new = fmaxf(m2, bmin * nq2);
        const float alpha = __builtin_amdgcn_exp2f(m2 - m_new);
        const float mm = m_new - LOG2_R_NORM;
        m2 = m_new;
        // line 11 for key tile `wave`
        v4i pw;
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
            float x[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) x[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(a[4 * vq + e], nq2, -mm));
            const uint32_t w = pack_p4(x);
            pw[vq] = static_cast<int>(w);
        }
        sm.p[wave][lane] = pw;
        wait_vmcnt<2 * PER_BLOCK>();                             // my pieces of block jb + 1 have landed (two later blocks may be in flight)
        __syncthreads();                                         // everyone's have, and every P tile of this block is in LDS
        // lines 12, 13: d tile `wave` of O^T = V^T P^T over the four key tiles, the row sum over the same P dwords
        if (wave >= KS) continue;                                // D = 64: two d tiles; the other wavefronts only take part above
        v16i pacc;
        uint32_t psum = 0;
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
            const v4i pf = sm.p[mt][lane];
            const v2i t0 = __builtin_amdgcn_ds_read_tr8_b64_v2i32(reinterpret_cast<LDS_AS v2i *>(v_operand<D>(vs, lo, wave) + 32 * mt * D));
            const v2i t1 = __builtin_amdgcn_ds_read_tr8_b64_v2i32(reinterpret_cast<LDS_AS v2i *>(v_operand<D>(vs, lo, wave) + 16 * D + 32 * mt * D));
            const v4i vop = {t0[0], t0[1], t1[0], t1[1]};
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) psum = __builtin_amdgcn_sad_u8(static_cast<uint32_t>(pf[vq]), 0u, psum);
            pacc = __builtin_amdgcn_mfma_i32_32x32x32_i8(vop, pf, mt == 0 ? acc0 : pacc, 0, 0, 0);
        }
        l = __builtin_fmaf(l, alpha, static_cast<float>(psum));
        const float alpha_o = VB ? alpha * oscale : alpha;
#pragma unroll
        for (int v = 0; v < 16; ++v) o[v] = __builtin_fmaf(o[v], alpha_o, -(ACC_START_F - __int_as_float(pacc[v])));
    }
    wait_all_memory();                                           // requests past the last block: nothing of mine stays in flight

    // lines 15-17 for d tile `wave` (d = 32 * wave + 8 * (v / 4) + 4 * g + v % 4 of query r)
    const float lt = l + swap32(l);
    const float f = (VB ? sv_prev : sVh[0]) * ACC_UNIT / lt;
    if (q_head < Nq && wave < KS) {
        OutT *orow = O + (static_cast<long>(head) * Nq + q_head) * D + 32 * wave + 4 * g;
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
            if constexpr (sizeof(OutT) == 2) {
                *reinterpret_cast<uint2 *>(orow + 8 * vq) = Pack4<OutT>::pack(o[4 * vq] * f, o[4 * vq + 1] * f, o[4 * vq + 2] * f, o[4 * vq + 3] * f);
            } else {
                *reinterpret_cast<v4f *>(orow + 8 * vq) = v4f{o[4 * vq] * f, o[4 * vq + 1] * f, o[4 * vq + 2] * f, o[4 * vq + 3] * f};
            }
        }
    }
#endif
}

// ---- few queries, many keys, any number of heads: the key axis split across workgroups, exactly ----------------
// One workgroup per head (the narrow kernel) cannot fill the chip when there are few heads, and even with 128 of them
// it is bound by its own block-to-block latency.  Splitting the keys of a head over workgroups is not Algorithm 1 as
// long as each part rounds P on the grid of ITS OWN running maximum; it is Algorithm 1 once the maximum after every
// key block is known before any P is formed.  With at most SPLIT_MAX_Q queries per head the scores are small next to
// K and V (4 N_q bytes per key against 2 d), so they go through memory:
//   pass 1 (splitk_scores_kernel)  streams K, computes line 9 exactly as the other kernels do (same MFMA chain, same
//           scaling) and writes the scaled scores a, the minimum of every (32-key tile, query) -- the maxima of line 10
//           -- and the minimum of every (run of blocks, query);
//   pass 2 (splitk_pv_kernel)      streams V and the scores; the running maximum in front of a workgroup's first block
//           is the extremum over all earlier runs (max is exact and order-independent), so lines 10-13 give, block by
//           block, the same m, the same P bytes and the same int32 P V as the sequential walk; what a workgroup leaves
//           is the walk over its run of blocks started from O = 0, l = 0: a partial (m, l, O);
//   pass 3 (splitk_combine_kernel) O = sum over the runs of 2^(m_run - m_last) O_run, l likewise, then lines 15-17.
// P is bit-identical to the sequential kernels'; O and l differ from theirs only in the order of the fp32 additions
// (the sequential walk multiplies by e^{m_old - m} block after block, this one once per partial).
// In both streaming passes a workgroup takes a run of `cb` key blocks of one head and its wavefront w takes key tile w
// (keys 32w .. 32w + 31) of each of them: the rows of K, V, s_K and of the scores that a wavefront stages into LDS
// are exactly the rows it consumes itself, so the wavefronts of a workgroup never wait for one another -- no barrier
// in the loops; a wavefront's ring of staged blocks is ordered by its own counted s_waitcnt alone.  The four
// wavefronts meet once, after their loops: their minima (pass 1) and their partial (l, O) at the common m (pass 2)
// are combined through LDS.
constexpr int SPLIT_MAX_Q = 8;       // queries per head up to which the scores go through memory (a decode step, a few speculative tokens)
constexpr int SPLIT_MAX_Q_RECOMPUTE = 32;   // ... and up to which the second pass recomputes them from K instead (one column tile)
constexpr int SPLIT_RECOMPUTE_MAX_HEADS = 96;   // ... as long as there are fewer heads than this
constexpr int SPLIT_NSTAGE_K = 4;    // pass 1: ring of K blocks, filled three ahead
constexpr int SPLIT_NSTAGE_V = 3;    // pass 2: ring of V blocks, filled two ahead
[[maybe_unused]] constexpr bool SPLIT_NT = true;      // staging copies carry the non-temporal hint: every byte is read once (measured +7 % at 537 MB of K and V)

template <int D> struct SmemSplitK {
    alignas(4096) int8_t k[SPLIT_NSTAGE_K][BC * D];
    alignas(256) float sk[SPLIT_NSTAGE_K][4][64];             // per wavefront: the 32 s_K of its key tile (+ 32 unused)
    alignas(16) float red[4][SPLIT_MAX_Q_RECOMPUTE];
};
template <int D> struct SmemSplitV {
    alignas(4096) int8_t v[SPLIT_NSTAGE_V][BC * D];
    alignas(1024) float a[SPLIT_NSTAGE_V][4][SPLIT_MAX_Q][32];   // per wavefront: the scores of its key tile, query-major
    alignas(256) float tmin[SPLIT_NSTAGE_V][4][64];             // per wavefront: the block's [query][tile] minima (+ 32 unused)
    alignas(16) float red[4][SPLIT_MAX_Q];
    alignas(16) float pre[SPLIT_MAX_Q];
};
static_assert(2 * sizeof(SmemSplitK<128>) <= 160 * 1024 && 2 * sizeof(SmemSplitV<128>) <= 160 * 1024, "two workgroups per CU");
static_assert(offsetof(SmemSplitV<64>, v) % 4096 == 0 && (BC * 64) % 4096 == 0, "tile bases");

// Second pass for 9 .. 32 queries per head: the scores would be as many bytes as K and V, so they are not stored;
// the pass streams K once more and recomputes line 9 (same MFMA chain, same scaling: the same numbers).
template <int D> struct SmemSplitKV {
    alignas(4096) int8_t k[SPLIT_NSTAGE_V][BC * D];
    alignas(4096) int8_t v[SPLIT_NSTAGE_V][BC * D];
    alignas(256) float sk[SPLIT_NSTAGE_V][4][64];
    alignas(1024) float tmin[SPLIT_NSTAGE_V][4][256];           // per wavefront: the block's [query][tile] minima (512 B, + 512 unused)
    alignas(16) float pre[SPLIT_MAX_Q_RECOMPUTE];
};
static_assert(sizeof(SmemSplitKV<128>) <= 160 * 1024, "LDS budget");

// Layout of the workspace (fp32 words), shared by the host code and the kernels (MAXQ = 8 or 32, by Nq):
//   scores  [heads, T_c, 4 tiles, Nq, 32]     a of line 9 (masked keys: +inf); Nq <= 8 only
//   tmin    [heads, T_c, MAXQ, 4]             minimum of a per (block, query, tile); queries >= Nq unused
//   cmin    [heads, MAXQ, nchunks]            minimum of a per (run of blocks, query)
//   part_o  [heads, parts, Nq, d]             one partial per run of blocks
//   part_ml [heads, parts, Nq, 2]             m (log2 units) and l of the partial
struct SplitPlan {
    int cb, nchunks, T_c, maxq, parts;
    bool store;
    long off_tmin, off_cmin, off_part_o, off_part_ml, words;
};
inline SplitPlan split_plan(long heads, int Nq, int Nk, int d) {
    SplitPlan p;
    p.T_c = (Nk + BC - 1) / BC;
    p.store = Nq <= SPLIT_MAX_Q;
    p.maxq = p.store ? SPLIT_MAX_Q : SPLIT_MAX_Q_RECOMPUTE;
    long want = 1024 / heads;                    // about four workgroups per CU over the chip
    if (want < 1) want = 1;
    long cb = (p.T_c + want - 1) / want;
    const long cb_min = p.store ? 2 : 4;         // a run's partial (Nq x d floats) must stay small next to its K and V
    if (cb < cb_min) cb = cb_min;
    if (cb > p.T_c) cb = p.T_c;
    p.cb = static_cast<int>(cb);
    p.nchunks = (p.T_c + p.cb - 1) / p.cb;       // no run is empty
    p.parts = p.nchunks;
    auto up = [](long w) { return (w + 63) & ~63L; };            // 256-byte granules
    p.off_tmin = p.store ? up(heads * p.T_c * 4 * Nq * 32) : 0;
    p.off_cmin = p.off_tmin + up(heads * p.T_c * p.maxq * 4);
    p.off_part_o = p.off_cmin + up(heads * p.maxq * p.nchunks);
    p.off_part_ml = p.off_part_o + up(heads * p.parts * Nq * d);
    p.words = p.off_part_ml + up(heads * p.parts * Nq * 2);
    return p;
}

template <int D, bool CAUSAL, int MAXQ, bool STORE>
__global__ __launch_bounds__(THREADS, 2) void splitk_scores_kernel(
    const int8_t *__restrict__ Q, const int8_t *__restrict__ K, const float *__restrict__ sK, int Nq, int Nk, int cb,
    int nchunks, float *__restrict__ scores, float *__restrict__ tminG, float *__restrict__ cminG) {
#if defined(__HIP_DEVICE_COMPILE__)
    __shared__ SmemSplitK<D> sm;
    constexpr int KS = D / 32;
    constexpr int PER_BLOCK = KS + 1;                            // copy instructions per wavefront and block
    const int tid = threadIdx.x, lane = tid & 63, r = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int T_c = (Nk + BC - 1) / BC;
    const int head = blockIdx.x / nchunks, c = blockIdx.x % nchunks;
    const int jb0 = c * cb, jb1 = min(T_c, jb0 + cb);            // this workgroup's key blocks
    const int shift = CAUSAL ? Nk - Nq : 0;
    const int rq = min(r, Nq - 1);                               // columns past Nq: a copy of the last query, never stored

    const BufRsrc rK = make_rsrc(K + static_cast<long>(head) * Nk * D, static_cast<unsigned>(Nk) * D);
    const BufRsrc rSK = make_rsrc(sK + static_cast<long>(head) * Nk, static_cast<unsigned>(Nk) * 4);
    const lds_ptr kbuf = (lds_ptr)(&sm.k[0][0]);
    const lds_ptr skbuf = (lds_ptr)(&sm.sk[0][0][0]);
    const LaneOffsets<D> lo(lane, wave);
    // Line 8 for this wavefront's key tile of block jb (rows 32 wave .. + 31 of K_j: the pieces prefetch_k_piece gives
    // this wavefront; its 32 s_K, lanes 32-63 repeating lanes 0-31) into stage (jb - jb0) % NSTAGE.  A block past the
    // run is requested nowhere, so that every block costs PER_BLOCK copy instructions and the counted waits stay valid.
    auto stage_block = [&](int jb) {
        const int st = (jb - jb0) % SPLIT_NSTAGE_K;
        const bool real = jb < jb1;
        const Prefetch pf = {rK, rK, rSK, real ? jb * BC * D : NOWHERE, real ? jb * BC * 4 : NOWHERE,
                             kbuf + st * BC * D, kbuf, skbuf + (st * 4 + wave) * 256};
#pragma unroll
        for (int i = 0; i < KS; ++i) prefetch_k_piece<D, SPLIT_NT>(pf, lo, wave, i);
        lds_copy4(pf.sk, pf.lsk, 4 * r + 128 * wave, pf.skoff);
    };
    stage_block(jb0);
    stage_block(jb0 + 1);
    stage_block(jb0 + 2);

    const int8_t *qptr = Q + (static_cast<long>(head) * Nq + rq) * D + 16 * g;
    v4i qf[KS];
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) qf[kk] = *reinterpret_cast<const v4i *>(qptr + 32 * kk);
    // landed BEFORE the loop as far as the compiler is concerned: a wait of its own inside the loop would be a wait for
    // every outstanding vector-memory operation, the staged copies included
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) asm volatile("" : "+v"(qf[kk]));
    v16i acc0;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc0[v] = ACC_START_I;
    float wmin = INFINITY;                                       // minimum over this wavefront's tiles of the whole run

    for (int jb = jb0; jb < jb1; ++jb) {
        const int st = (jb - jb0) % SPLIT_NSTAGE_K, j0 = jb * BC;
        // The counter retires in order.  Younger than the copies of block jb are those of blocks jb + 1 and jb + 2 and
        // the stores of earlier iterations: allowing 2 PER_BLOCK operations in flight means block jb has landed,
        // however many stores there are among them.
        wait_vmcnt<2 * PER_BLOCK>();
        stage_block(jb + 3);                                     // into the stage of block jb - 1, which this wavefront has left
        const lds_ptr ks = kbuf + st * BC * D;
        v4i kop[KS];
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) kop[kk] = *reinterpret_cast<LDS_AS const v4i *>(k_operand<D>(ks, lo, kk) + 32 * wave * D);
        v4f skv[4];
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) skv[vq] = *reinterpret_cast<LDS_AS const v4f *>(skbuf + (st * 4 + wave) * 256 + lo.sk + 32 * vq);
        v16i sacc = acc0;
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) sacc = __builtin_amdgcn_mfma_i32_32x32x32_i8(kop[kk], qf[kk], sacc, 0, 0, 0);
        // kept keys: index inside the block <= klimit (the causal diagonal, the ragged end of the sequence)
        const int tail = Nk - 1 - j0;
        const int klimit = CAUSAL ? min(rq + shift - j0, tail) : tail;
        const bool masked = CAUSAL ? (j0 + BC - 1 > min(shift, Nk - 1)) : (tail < BC - 1);   // wave-uniform
        float a[16], tmin = INFINITY;
#pragma unroll
        for (int vq = 0; vq < 4; ++vq)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float x = (ACC_START_F - __int_as_float(sacc[4 * vq + e])) * skv[vq][e];
                if (masked && (32 * wave + 8 * vq + 4 * g + e > klimit)) x = INFINITY;
                a[4 * vq + e] = x;
                tmin = fminf(tmin, x);
            }
        tmin = pair_min(tmin);
        wmin = fminf(wmin, tmin);
        if (r < Nq) {
            if (STORE) {
                float *dst = scores + (((static_cast<long>(head) * T_c + jb) * 4 + wave) * Nq + r) * 32 + 4 * g;
#pragma unroll
                for (int vq = 0; vq < 4; ++vq) *reinterpret_cast<v4f *>(dst + 8 * vq) = v4f{a[4 * vq], a[4 * vq + 1], a[4 * vq + 2], a[4 * vq + 3]};
            }
            if (g == 0) tminG[((static_cast<long>(head) * T_c + jb) * MAXQ + r) * 4 + wave] = tmin;
        }
    }
    wait_all_memory();                                           // requests past the run: nothing of mine stays in flight
    // the run's minimum per query, for the prefix the second pass needs: the only exchange between the wavefronts
    if (g == 0 && r < MAXQ) sm.red[wave][r] = wmin;
    __syncthreads();
    if (wave == 0 && g == 0 && r < Nq)
        cminG[(static_cast<long>(head) * MAXQ + r) * nchunks + c] = fminf(fminf(sm.red[0][r], sm.red[1][r]), fminf(sm.red[2][r], sm.red[3][r]));
#endif
}

template <int D>
__global__ __launch_bounds__(THREADS, 2) void splitk_pv_kernel(
    const int8_t *__restrict__ V, const float *__restrict__ sQ, int Nq, int Nk, int cb, int nchunks,
    const float *__restrict__ scores, const float *__restrict__ tminG, const float *__restrict__ cminG, float *__restrict__ part_o,
    float *__restrict__ part_ml) {
#if defined(__HIP_DEVICE_COMPILE__)
    __shared__ SmemSplitV<D> sm;
    constexpr int DT = D / 32;
    constexpr int PER_BLOCK = DT + 2;
    const int tid = threadIdx.x, lane = tid & 63, r = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int T_c = (Nk + BC - 1) / BC;
    const int head = blockIdx.x / nchunks, c = blockIdx.x % nchunks;
    const int jb0 = c * cb, jb1 = min(T_c, jb0 + cb);
    const int rq = min(r, Nq - 1);

    const BufRsrc rV = make_rsrc(V + static_cast<long>(head) * Nk * D, static_cast<unsigned>(Nk) * D);
    const BufRsrc rA = make_rsrc(scores + static_cast<long>(head) * T_c * 4 * Nq * 32, static_cast<unsigned>(T_c) * 4 * Nq * 32 * 4);
    const BufRsrc rT = make_rsrc(tminG + static_cast<long>(head) * T_c * SPLIT_MAX_Q * 4, static_cast<unsigned>(T_c) * SPLIT_MAX_Q * 4 * 4);
    const lds_ptr vbuf = (lds_ptr)(&sm.v[0][0]);
    const lds_ptr abuf = (lds_ptr)(&sm.a[0][0][0][0]);
    const lds_ptr tbuf = (lds_ptr)(&sm.tmin[0][0][0]);
    const LaneOffsets<D> lo(lane, wave);
    // This wavefront's key tile of V_j (the rows prefetch_v_piece gives it), the scores of that tile (Nq x 32 floats,
    // contiguous; the copy moves 1 KB, whatever follows the record is not read) and the block's 32 tile minima.
    auto stage_block = [&](int jb) {
        const int st = (jb - jb0) % SPLIT_NSTAGE_V;
        const bool real = jb < jb1;
        const Prefetch pf = {rV, rV, rV, real ? jb * BC * D : NOWHERE, NOWHERE, vbuf, vbuf + st * BC * D, vbuf};
#pragma unroll
        for (int i = 0; i < DT; ++i) prefetch_v_piece<D, SPLIT_NT>(pf, lo, wave, i);
        lds_copy16(rA, abuf + (st * 4 + wave) * 1024, 16 * lane, real ? (jb * 4 + wave) * Nq * 128 : NOWHERE);
        lds_copy4(rT, tbuf + (st * 4 + wave) * 256, 4 * r, real ? jb * (SPLIT_MAX_Q * 4 * 4) : NOWHERE);
    };
    stage_block(jb0);
    stage_block(jb0 + 1);

    float nq2 = sQ[static_cast<long>(head) * Nq + rq] * (-LOG2E * ACC_UNIT);
    // Minimum of a over every block in front of this workgroup's first one: over the runs in front of this one.
    // 32 threads per query (wavefront w: queries 2w and 2w + 1).
    float pre = INFINITY;
    {
        const int q = tid >> 5;
        if (q < Nq)
            for (int cc = tid & 31; cc < c; cc += 32) pre = fminf(pre, cminG[(static_cast<long>(head) * SPLIT_MAX_Q + q) * nchunks + cc]);
#pragma unroll
        for (int s_ = 16; s_ >= 1; s_ >>= 1) pre = fminf(pre, __shfl_xor(pre, s_));
        if ((tid & 31) == 0) sm.pre[q] = pre;
    }
    asm volatile("" : "+v"(nq2));                                // as for Q above: no wait of the compiler's own inside the loop
    __syncthreads();
    pre = sm.pre[rq];
    float m2 = (pre == INFINITY) ? -INFINITY : pre * nq2;        // line 10 over all earlier blocks (no block: line 6)
    float l = 0.0f, o[DT][16];
    v16i acc0;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        acc0[v] = ACC_START_I;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) o[dt][v] = 0.0f;
    }

    for (int jb = jb0; jb < jb1; ++jb) {
        const int st = (jb - jb0) % SPLIT_NSTAGE_V;
        wait_vmcnt<PER_BLOCK>();                                 // block jb has landed (block jb + 1 may be in flight)
        stage_block(jb + 2);                                     // into the stage of block jb - 1, which this wavefront has left
        const lds_ptr vs = vbuf + st * BC * D;
        // line 10 for the whole block: the four tile minima of this lane's query
        const v4f t4 = *reinterpret_cast<LDS_AS const v4f *>(tbuf + (st * 4 + wave) * 256 + rq * 16);
        const float bmin = fminf(fminf(t4[0], t4[1]), fminf(t4[2], t4[3]));
        const float m_new = fmaxf(m2, bmin * nq2);
        const float alpha = __builtin_amdgcn_exp2f(m2 - m_new);
        const float mm = m_new - LOG2_R_NORM;
        m2 = m_new;
        // line 11 for key tile `wave`
        v4i pw;
        uint32_t psum = 0;
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
            const v4f av = *reinterpret_cast<LDS_AS const v4f *>(abuf + (st * 4 + wave) * 1024 + rq * 128 + (8 * vq + 4 * g) * 4);
            float x[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) x[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(av[e], nq2, -mm));
            const uint32_t w = pack_p4(x);
            psum = __builtin_amdgcn_sad_u8(w, 0u, psum);
            pw[vq] = static_cast<int>(w);
        }
        l = __builtin_fmaf(l, alpha, static_cast<float>(psum));  // line 12 over this lane's keys of this tile
        // line 13 over the keys of this tile, all d tiles
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            const v2i t0 = __builtin_amdgcn_ds_read_tr8_b64_v2i32(reinterpret_cast<LDS_AS v2i *>(v_operand<D>(vs, lo, dt) + 32 * wave * D));
            const v2i t1 = __builtin_amdgcn_ds_read_tr8_b64_v2i32(reinterpret_cast<LDS_AS v2i *>(v_operand<D>(vs, lo, dt) + 16 * D + 32 * wave * D));
            const v4i vop = {t0[0], t0[1], t1[0], t1[1]};
            const v16i pacc = __builtin_amdgcn_mfma_i32_32x32x32_i8(vop, pw, acc0, 0, 0, 0);
#pragma unroll
            for (int v = 0; v < 16; ++v) o[dt][v] = __builtin_fmaf(o[dt][v], alpha, -(ACC_START_F - __int_as_float(pacc[v])));
        }
    }
    wait_all_memory();
    // The four wavefronts hold partials of the same run of blocks at the same m: their sum is the workgroup's partial.
    // The V ring is free once every wavefront has left the loop; [wavefront][query][d] floats go through it.
    const float lt = l + swap32(l);
    __syncthreads();
    float *xo = reinterpret_cast<float *>(&sm.v[0][0]);          // 4 * 8 * D floats <= 16 KB
    if (r < Nq) {
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int vq = 0; vq < 4; ++vq)
                *reinterpret_cast<v4f *>(xo + (wave * SPLIT_MAX_Q + r) * D + 32 * dt + 8 * vq + 4 * g) = v4f{o[dt][4 * vq], o[dt][4 * vq + 1], o[dt][4 * vq + 2], o[dt][4 * vq + 3]};
        if (g == 0) sm.red[wave][r] = lt;
    }
    __syncthreads();
    const long slot0 = (static_cast<long>(head) * nchunks + c) * Nq;
    for (int idx = tid; idx < Nq * D; idx += THREADS) {
        const int q = idx / D, t = idx % D;
        part_o[(slot0 + q) * D + t] = (xo[(0 * SPLIT_MAX_Q + q) * D + t] + xo[(1 * SPLIT_MAX_Q + q) * D + t]) +
                                      (xo[(2 * SPLIT_MAX_Q + q) * D + t] + xo[(3 * SPLIT_MAX_Q + q) * D + t]);
    }
    if (wave == 0 && g == 0 && r < Nq) {
        part_ml[2 * (slot0 + r)] = m2;
        part_ml[2 * (slot0 + r) + 1] = (sm.red[0][r] + sm.red[1][r]) + (sm.red[2][r] + sm.red[3][r]);
    }
#endif
}

// Second pass for 9 .. 32 queries per head (see SmemSplitKV): lines 9-13 per key tile with m known beforehand.
template <int D, bool CAUSAL>
__global__ __launch_bounds__(THREADS, 1) void splitk_pv_recompute_kernel(
    const int8_t *__restrict__ Q, const int8_t *__restrict__ K, const int8_t *__restrict__ V, const float *__restrict__ sQ,
    const float *__restrict__ sK, int Nq, int Nk, int cb, int nchunks, const float *__restrict__ tminG,
    const float *__restrict__ cminG, float *__restrict__ part_o, float *__restrict__ part_ml) {
#if defined(__HIP_DEVICE_COMPILE__)
    __shared__ SmemSplitKV<D> sm;
    constexpr int KS = D / 32, DT = D / 32, MAXQ = SPLIT_MAX_Q_RECOMPUTE;
    constexpr int PER_BLOCK = KS + DT + 2;                       // copy instructions per wavefront and block
    const int tid = threadIdx.x, lane = tid & 63, r = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int T_c = (Nk + BC - 1) / BC;
    const int head = blockIdx.x / nchunks, c = blockIdx.x % nchunks;
    const int jb0 = c * cb, jb1 = min(T_c, jb0 + cb);
    const int shift = CAUSAL ? Nk - Nq : 0;
    const int rq = min(r, Nq - 1);

    const BufRsrc rK = make_rsrc(K + static_cast<long>(head) * Nk * D, static_cast<unsigned>(Nk) * D);
    const BufRsrc rV = make_rsrc(V + static_cast<long>(head) * Nk * D, static_cast<unsigned>(Nk) * D);
    const BufRsrc rSK = make_rsrc(sK + static_cast<long>(head) * Nk, static_cast<unsigned>(Nk) * 4);
    const BufRsrc rT = make_rsrc(tminG + static_cast<long>(head) * T_c * MAXQ * 4, static_cast<unsigned>(T_c) * MAXQ * 4 * 4);
    const lds_ptr kbuf = (lds_ptr)(&sm.k[0][0]);
    const lds_ptr vbuf = (lds_ptr)(&sm.v[0][0]);
    const lds_ptr skbuf = (lds_ptr)(&sm.sk[0][0][0]);
    const lds_ptr tbuf = (lds_ptr)(&sm.tmin[0][0][0]);
    const LaneOffsets<D> lo(lane, wave);
    // this wavefront's key tile of K_j and V_j, its 32 s_K, and the block's 128 tile minima (lanes 32-63 repeat 0-31)
    auto stage_block = [&](int jb) {
        const int st = (jb - jb0) % SPLIT_NSTAGE_V;
        const bool real = jb < jb1;
        const Prefetch pf = {rK, rV, rSK, real ? jb * BC * D : NOWHERE, real ? jb * BC * 4 : NOWHERE,
                             kbuf + st * BC * D, vbuf + st * BC * D, skbuf + (st * 4 + wave) * 256};
#pragma unroll
        for (int i = 0; i < KS; ++i) prefetch_k_piece<D, SPLIT_NT>(pf, lo, wave, i);
#pragma unroll
        for (int i = 0; i < DT; ++i) prefetch_v_piece<D, SPLIT_NT>(pf, lo, wave, i);
        lds_copy4(pf.sk, pf.lsk, 4 * r + 128 * wave, pf.skoff);
        lds_copy16(rT, tbuf + (st * 4 + wave) * 1024, 16 * r, real ? jb * (MAXQ * 4 * 4) : NOWHERE);
    };
    stage_block(jb0);
    stage_block(jb0 + 1);

    const int8_t *qptr = Q + (static_cast<long>(head) * Nq + rq) * D + 16 * g;
    v4i qf[KS];
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) qf[kk] = *reinterpret_cast<const v4i *>(qptr + 32 * kk);
    float nq2 = sQ[static_cast<long>(head) * Nq + rq] * (-LOG2E * ACC_UNIT);
    // minimum of a over the runs in front of this one: 8 threads per query
    float pre = INFINITY;
    {
        const int q = tid >> 3;
        if (q < Nq)
            for (int cc = tid & 7; cc < c; cc += 8) pre = fminf(pre, cminG[(static_cast<long>(head) * MAXQ + q) * nchunks + cc]);
#pragma unroll
        for (int s_ = 4; s_ >= 1; s_ >>= 1) pre = fminf(pre, __shfl_xor(pre, s_));
        if ((tid & 7) == 0) sm.pre[q] = pre;
    }
    // landed BEFORE the loop as far as the compiler is concerned (no wait of its own for them inside the loop)
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) asm volatile("" : "+v"(qf[kk]));
    asm volatile("" : "+v"(nq2));
    __syncthreads();
    pre = sm.pre[rq];
    float m2 = (pre == INFINITY) ? -INFINITY : pre * nq2;        // line 10 over all earlier blocks (no block: line 6)
    float l = 0.0f, o[DT][16];
    v16i acc0;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        acc0[v] = ACC_START_I;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) o[dt][v] = 0.0f;
    }

    for (int jb = jb0; jb < jb1; ++jb) {
        const int st = (jb - jb0) % SPLIT_NSTAGE_V, j0 = jb * BC;
        wait_vmcnt<PER_BLOCK>();                                 // block jb has landed (block jb + 1 may be in flight)
        stage_block(jb + 2);                                     // into the stage of block jb - 1, which this wavefront has left
        const lds_ptr ks = kbuf + st * BC * D, vs = vbuf + st * BC * D;
        // line 9 for key tile `wave`, as in the first pass
        v4i kop[KS];
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) kop[kk] = *reinterpret_cast<LDS_AS const v4i *>(k_operand<D>(ks, lo, kk) + 32 * wave * D);
        v4f skv[4];
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) skv[vq] = *reinterpret_cast<LDS_AS const v4f *>(skbuf + (st * 4 + wave) * 256 + lo.sk + 32 * vq);
        v16i sacc = acc0;
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) sacc = __builtin_amdgcn_mfma_i32_32x32x32_i8(kop[kk], qf[kk], sacc, 0, 0, 0);
        const int tail = Nk - 1 - j0;
        const int klimit = CAUSAL ? min(rq + shift - j0, tail) : tail;
        const bool masked = CAUSAL ? (j0 + BC - 1 > min(shift, Nk - 1)) : (tail < BC - 1);   // wave-uniform
        // line 10 for the whole block: the four tile minima of this lane's query
        const v4f t4 = *reinterpret_cast<LDS_AS const v4f *>(tbuf + (st * 4 + wave) * 1024 + rq * 16);
        const float bmin = fminf(fminf(t4[0], t4[1]), fminf(t4[2], t4[3]));
        const float m_new = fmaxf(m2, bmin * nq2);
        const float alpha = __builtin_amdgcn_exp2f(m2 - m_new);
        const float mm = m_new - LOG2_R_NORM;
        m2 = m_new;
        // line 11
        v4i pw;
        uint32_t psum = 0;
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
            float x[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float av = (ACC_START_F - __int_as_float(sacc[4 * vq + e])) * skv[vq][e];
                if (masked && (32 * wave + 8 * vq + 4 * g + e > klimit)) av = INFINITY;
                x[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(av, nq2, -mm));
            }
            const uint32_t w = pack_p4(x);
            psum = __builtin_amdgcn_sad_u8(w, 0u, psum);
            pw[vq] = static_cast<int>(w);
        }
        l = __builtin_fmaf(l, alpha, static_cast<float>(psum));  // line 12 over this lane's keys of this tile
        // line 13 over the keys of this tile, all d tiles
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            const v2i t0 = __builtin_amdgcn_ds_read_tr8_b64_v2i32(reinterpret_cast<LDS_AS v2i *>(v_operand<D>(vs, lo, dt) + 32 * wave * D));
            const v2i t1 = __builtin_amdgcn_ds_read_tr8_b64_v2i32(reinterpret_cast<LDS_AS v2i *>(v_operand<D>(vs, lo, dt) + 16 * D + 32 * wave * D));
            const v4i vop = {t0[0], t0[1], t1[0], t1[1]};
            const v16i pacc = __builtin_amdgcn_mfma_i32_32x32x32_i8(vop, pw, acc0, 0, 0, 0);
#pragma unroll
            for (int v = 0; v < 16; ++v) o[dt][v] = __builtin_fmaf(o[dt][v], alpha, -(ACC_START_F - __int_as_float(pacc[v])));
        }
    }
    wait_all_memory();
    // The four wavefronts hold partials of the same run at the same m: their sum is the workgroup's partial.  The K
    // and V rings (contiguous) are free once every wavefront has left the loop; [wavefront][query][d] floats go through them.
    static_assert(offsetof(SmemSplitKV<D>, v) == sizeof(SmemSplitKV<D>::k) && 4 * MAXQ * D * 4 <= 2 * SPLIT_NSTAGE_V * BC * D, "exchange area");
    const float lt = l + swap32(l);
    __syncthreads();
    float *xo = reinterpret_cast<float *>(&sm.k[0][0]);
    float *xl = reinterpret_cast<float *>(&sm.sk[0][0][0]);      // [wavefront][query]
    if (r < Nq) {
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int vq = 0; vq < 4; ++vq)
                *reinterpret_cast<v4f *>(xo + (wave * MAXQ + r) * D + 32 * dt + 8 * vq + 4 * g) = v4f{o[dt][4 * vq], o[dt][4 * vq + 1], o[dt][4 * vq + 2], o[dt][4 * vq + 3]};
        if (g == 0) xl[wave * MAXQ + r] = lt;
    }
    __syncthreads();
    const long slot0 = (static_cast<long>(head) * nchunks + c) * Nq;
    for (int idx = tid; idx < Nq * D; idx += THREADS) {
        const int q = idx / D, t = idx % D;
        part_o[(slot0 + q) * D + t] = (xo[(0 * MAXQ + q) * D + t] + xo[(1 * MAXQ + q) * D + t]) + (xo[(2 * MAXQ + q) * D + t] + xo[(3 * MAXQ + q) * D + t]);
    }
    if (wave == 0 && g == 0 && r < Nq) {
        part_ml[2 * (slot0 + r)] = m2;
        part_ml[2 * (slot0 + r) + 1] = (xl[r] + xl[MAXQ + r]) + (xl[2 * MAXQ + r] + xl[3 * MAXQ + r]);
    }
#endif
}

// Lines 15-17 over the partial results of one (head, query).  256 threads: thread (pg, dq) sums the parts p = pg, pg + PG,
// ... for output columns 4 dq .. 4 dq + 3 (PG = 1024 / D groups of parts, D / 4 column quads), LDS adds the groups up.
template <int D, typename OutT>
__global__ __launch_bounds__(THREADS) void splitk_combine_kernel(const float *__restrict__ part_o, const float *__restrict__ part_ml,
                                                                 const float *__restrict__ sV, int Nq, int parts, OutT *__restrict__ O) {
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr int DQ = D / 4, PG = THREADS / DQ;
    __shared__ float xo[PG][D];
    __shared__ float xl[PG];
    const long hq = blockIdx.x, head = hq / Nq, q = hq % Nq;
    const int dq = threadIdx.x % DQ, pg = threadIdx.x / DQ;
    const long slot0 = head * parts * Nq + q;
    const float m_last = part_ml[2 * (slot0 + static_cast<long>(parts - 1) * Nq)];   // the running maximum never decreases
    v4f acc = {0.0f, 0.0f, 0.0f, 0.0f};
    float l = 0.0f;
    for (int p = pg; p < parts; p += PG) {
        const long slot = slot0 + static_cast<long>(p) * Nq;
        const float w = __builtin_amdgcn_exp2f(part_ml[2 * slot] - m_last);
        const v4f x = *reinterpret_cast<const v4f *>(part_o + slot * D + 4 * dq);
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] = __builtin_fmaf(x[e], w, acc[e]);
        l = __builtin_fmaf(part_ml[2 * slot + 1], w, l);
    }
    *reinterpret_cast<v4f *>(&xo[pg][4 * dq]) = acc;
    if (dq == 0) xl[pg] = l;
    __syncthreads();
    if (threadIdx.x < D) {
        const int t = threadIdx.x;
        float y = 0.0f, lsum = 0.0f;
#pragma unroll
        for (int i = 0; i < PG; ++i) { y += xo[i][t]; lsum += xl[i]; }
        y *= sV[head] * ACC_UNIT / lsum;
        asm volatile("" : "+v"(y));   // the fp32 product, rounded once more below: never a mixed-precision multiply that rounds straight to 16 bits
        if constexpr (sizeof(OutT) == 2) reinterpret_cast<uint16_t *>(O)[hq * D + t] = static_cast<uint16_t>(Pack4<OutT>::pack(y, 0.0f, 0.0f, 0.0f).x & 0xffffu);
        else O[hq * D + t] = y;
    }
#endif
}

// ---- host side ----------------------------------------------------------------------------------
template <int D, bool CAUSAL, bool VB, typename OutT>
int launch_narrow(const int8_t *Q, const int8_t *K, const int8_t *V, const float *sQ, const float *sK, const float *sV,
                  int heads, int Nq, int Nk, void *O, hipStream_t st) {
    const long wgs = static_cast<long>(heads) * ((Nq + NARROW_BR - 1) / NARROW_BR);
    hipLaunchKernelGGL((int_flash_attn_fwd_narrow_kernel<D, CAUSAL, VB, OutT>), dim3(static_cast<unsigned>(wgs)), dim3(THREADS), 0, st,
                       Q, K, V, sQ, sK, sV, heads, Nq, Nk, static_cast<OutT *>(O));
    return hipGetLastError() == hipSuccess ? IFA_OK : IFA_ERR_HIP;
}

// The three passes of the key-split path on one stream; `ws` is the workspace laid out by split_plan().
template <int D, bool CAUSAL, typename OutT>
int launch_splitk(const int8_t *Q, const int8_t *K, const int8_t *V, const float *sQ, const float *sK, const float *sV,
                  int heads, int Nq, int Nk, void *O, float *ws, hipStream_t st) {
    const SplitPlan p = split_plan(heads, Nq, Nk, D);
    float *scores = ws, *tmin = ws + p.off_tmin, *cmin = ws + p.off_cmin, *part_o = ws + p.off_part_o, *part_ml = ws + p.off_part_ml;
    const dim3 grid(static_cast<unsigned>(static_cast<long>(heads) * p.nchunks));
    if (p.store) {
        hipLaunchKernelGGL((splitk_scores_kernel<D, CAUSAL, SPLIT_MAX_Q, true>), grid, dim3(THREADS), 0, st, Q, K, sK, Nq, Nk, p.cb, p.nchunks,
                           scores, tmin, cmin);
        hipLaunchKernelGGL((splitk_pv_kernel<D>), grid, dim3(THREADS), 0, st, V, sQ, Nq, Nk, p.cb, p.nchunks, scores, tmin, cmin, part_o, part_ml);
    } else {
        hipLaunchKernelGGL((splitk_scores_kernel<D, CAUSAL, SPLIT_MAX_Q_RECOMPUTE, false>), grid, dim3(THREADS), 0, st, Q, K, sK, Nq, Nk, p.cb,
                           p.nchunks, scores, tmin, cmin);
        hipLaunchKernelGGL((splitk_pv_recompute_kernel<D, CAUSAL>), grid, dim3(THREADS), 0, st, Q, K, V, sQ, sK, Nq, Nk, p.cb, p.nchunks, tmin,
                           cmin, part_o, part_ml);
    }
    hipLaunchKernelGGL((splitk_combine_kernel<D, OutT>), dim3(static_cast<unsigned>(heads * Nq)), dim3(THREADS), 0, st, part_o, part_ml, sV,
                       Nq, p.parts, static_cast<OutT *>(O));
    return hipGetLastError() == hipSuccess ? IFA_OK : IFA_ERR_HIP;
}

template <int D, bool CAUSAL>
int launch_splitk_dtype(const int8_t *Q, const int8_t *K, const int8_t *V, const float *sQ, const float *sK, const float *sV,
                        int heads, int Nq, int Nk, void *O, int o_dtype, float *ws, hipStream_t st) {
    switch (o_dtype) {
    case IFA_F32: return launch_splitk<D, CAUSAL, float>(Q, K, V, sQ, sK, sV, heads, Nq, Nk, O, ws, st);
    case IFA_F16: return launch_splitk<D, CAUSAL, __half>(Q, K, V, sQ, sK, sV, heads, Nq, Nk, O, ws, st);
    default: return launch_splitk<D, CAUSAL, __hip_bfloat16>(Q, K, V, sQ, sK, sV, heads, Nq, Nk, O, ws, st);
    }
}

// argument checks of the key-split path that do not concern the workspace
int splitk_args(const signed char *Q_i8, const signed char *K_i8, const signed char *V_i8, const float *s_Q, const float *s_K,
                const float *s_V, int B, int H, int Nq, int Nk, int d, int causal, const void *O, int o_dtype) {
    if (!Q_i8 || !K_i8 || !V_i8 || !s_Q || !s_K || !s_V || !O) return IFA_ERR_NULL;
    if (B <= 0 || H <= 0 || Nq <= 0 || Nk <= 0 || d <= 0) return IFA_ERR_SHAPE;
    const long heads = static_cast<long>(B) * H;
    if (heads > (1L << 40) / Nk / d) return IFA_ERR_SHAPE;
    if (causal && Nk < Nq) return IFA_ERR_UNSUPPORTED;           // a query with no visible key
    if (o_dtype < IFA_F32 || o_dtype > IFA_BF16) return IFA_ERR_DTYPE;
    if ((d != 64 && d != 128) || Nq > SPLIT_MAX_Q_RECOMPUTE) return IFA_ERR_UNSUPPORTED;
    if (static_cast<long>(Nk) * d > 0x7ff00000L) return IFA_ERR_UNSUPPORTED;      // a head's K (or V) stays below NOWHERE
    const SplitPlan p = split_plan(heads, Nq, Nk, d);
    if (static_cast<long>(p.T_c) * 4 * p.maxq * 128 > 0x7ff00000L ||               // so do a head's scores and minima arrays
        heads * p.nchunks > 0x7fffffffL || heads * Nq > 0x7fffffffL) return IFA_ERR_UNSUPPORTED;
    if (!ifa_aligned16(Q_i8) || !ifa_aligned16(K_i8) || !ifa_aligned16(V_i8) || !ifa_aligned16(O) ||
        (reinterpret_cast<uintptr_t>(s_Q) & 3) || (reinterpret_cast<uintptr_t>(s_K) & 3) || (reinterpret_cast<uintptr_t>(s_V) & 3))
        return IFA_ERR_UNSUPPORTED;
    return IFA_OK;
}

int splitk_dispatch(const signed char *Q_i8, const signed char *K_i8, const signed char *V_i8, const float *s_Q, const float *s_K,
                    const float *s_V, int B, int H, int Nq, int Nk, int d, int causal, void *O, int o_dtype, float *ws,
                    hipStream_t st) {
    const int8_t *Q = reinterpret_cast<const int8_t *>(Q_i8);
    const int8_t *K = reinterpret_cast<const int8_t *>(K_i8);
    const int8_t *V = reinterpret_cast<const int8_t *>(V_i8);
    const int hd = B * H;
    // From 9 queries on the second pass reads K again: with many heads the one-workgroup-per-head kernel already fills the
    // chip and is the faster one (measured: 128 heads x 32 queries x 16384 keys 148 us against 167 us; 32 heads 160 against 73).
    if (Nq > SPLIT_MAX_Q && hd >= SPLIT_RECOMPUTE_MAX_HEADS)
        return int_flash_attn_fwd_rect(Q_i8, K_i8, V_i8, s_Q, s_K, s_V, B, H, Nq, Nk, d, causal, O, o_dtype, st);
    if (d == 128)
        return causal ? launch_splitk_dtype<128, true>(Q, K, V, s_Q, s_K, s_V, hd, Nq, Nk, O, o_dtype, ws, st)
                      : launch_splitk_dtype<128, false>(Q, K, V, s_Q, s_K, s_V, hd, Nq, Nk, O, o_dtype, ws, st);
    return causal ? launch_splitk_dtype<64, true>(Q, K, V, s_Q, s_K, s_V, hd, Nq, Nk, O, o_dtype, ws, st)
                  : launch_splitk_dtype<64, false>(Q, K, V, s_Q, s_K, s_V, hd, Nq, Nk, O, o_dtype, ws, st);
}

}  // namespace

// The narrow kernel for the dispatcher of the fused kernel's entry points (arguments already validated there).
int ifa_launch_narrow(const int8_t *Q, const int8_t *K, const int8_t *V, const float *sQ, const float *sK, const float *sV, int heads,
                      int Nq, int Nk, int d, int causal, int vblock, void *O, int o_dtype, hipStream_t st) {
    auto by_dtype = [&](auto D_, auto C_, auto VB_) {
        constexpr int D = decltype(D_)::value;
        constexpr bool C = decltype(C_)::value, VB = decltype(VB_)::value;
        switch (o_dtype) {
        case IFA_F32: return launch_narrow<D, C, VB, float>(Q, K, V, sQ, sK, sV, heads, Nq, Nk, O, st);
        case IFA_F16: return launch_narrow<D, C, VB, __half>(Q, K, V, sQ, sK, sV, heads, Nq, Nk, O, st);
        default: return launch_narrow<D, C, VB, __hip_bfloat16>(Q, K, V, sQ, sK, sV, heads, Nq, Nk, O, st);
        }
    };
    using I64 = std::integral_constant<int, 64>;
    using I128 = std::integral_constant<int, 128>;
    auto by_flags = [&](auto D_) {
        if (causal) return vblock ? by_dtype(D_, std::true_type{}, std::true_type{}) : by_dtype(D_, std::true_type{}, std::false_type{});
        return vblock ? by_dtype(D_, std::false_type{}, std::true_type{}) : by_dtype(D_, std::false_type{}, std::false_type{});
    };
    return d == 128 ? by_flags(I128{}) : by_flags(I64{});
}

extern "C" long ifa_splitk_workspace_bytes(int B, int H, int Nq, int Nk, int d) {
    if (B <= 0 || H <= 0 || Nq <= 0 || Nk <= 0 || (d != 64 && d != 128) || Nq > SPLIT_MAX_Q_RECOMPUTE) return 0;
    const long heads = static_cast<long>(B) * H;
    if (heads > (1L << 40) / Nk / d) return 0;
    return split_plan(heads, Nq, Nk, d).words * 4;
}

extern "C" int int_flash_attn_fwd_splitk(const signed char *Q_i8, const signed char *K_i8, const signed char *V_i8,
                                         const float *s_Q, const float *s_K, const float *s_V, int B, int H, int Nq, int Nk,
                                         int d, int causal, void *O, int o_dtype, void *workspace, long workspace_bytes,
                                         void *hip_stream) {
    const int rc = splitk_args(Q_i8, K_i8, V_i8, s_Q, s_K, s_V, B, H, Nq, Nk, d, causal, O, o_dtype);
    if (rc != IFA_OK) return rc;
    if (!workspace) return IFA_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(workspace) & 255) return IFA_ERR_UNSUPPORTED;
    if (workspace_bytes < ifa_splitk_workspace_bytes(B, H, Nq, Nk, d)) return IFA_ERR_WORKSPACE;
    return splitk_dispatch(Q_i8, K_i8, V_i8, s_Q, s_K, s_V, B, H, Nq, Nk, d, causal, O, o_dtype, static_cast<float *>(workspace),
                           static_cast<hipStream_t>(hip_stream));
}

// ---- the key-split path for callers that cannot allocate -------------------------------------------------------
// The same three launches with the workspace in a file-scope device array instead of a buffer of the caller's.  In
// host code the array's name is only a stand-in for the symbol: the device address is asked for once per device
// (hipGetSymbolAddress, with that device current) and kept; every GPU holds its own copy of the array.
constexpr long STATIC_WORKSPACE_BYTES = 16L << 20;
static __device__ __align__(256) unsigned char scratch[STATIC_WORKSPACE_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
void *g_scratch_ptr[MAX_DEVICES];
std::mutex g_scratch_mutex;

// device address of `scratch` on the current device, or null
void *static_workspace() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}
}  // namespace

// Also the set-up call: it resolves the array's address on the current device, so that a later
// int_flash_attn_fwd_splitk_static on this device (under graph capture, say) has no set-up left to do.
extern "C" long ifa_static_workspace_bytes(void) {
    (void)static_workspace();
    return STATIC_WORKSPACE_BYTES;
}

extern "C" int int_flash_attn_fwd_splitk_static(const signed char *Q_i8, const signed char *K_i8, const signed char *V_i8,
                                                const float *s_Q, const float *s_K, const float *s_V, int B, int H, int Nq,
                                                int Nk, int d, int causal, void *O, int o_dtype, void *hip_stream) {
    const int rc = splitk_args(Q_i8, K_i8, V_i8, s_Q, s_K, s_V, B, H, Nq, Nk, d, causal, O, o_dtype);
    if (rc != IFA_OK) return rc;
    if (ifa_splitk_workspace_bytes(B, H, Nq, Nk, d) > STATIC_WORKSPACE_BYTES) return IFA_ERR_WORKSPACE;
    void *ws = static_workspace();
    if (!ws) return IFA_ERR_HIP;
    return splitk_dispatch(Q_i8, K_i8, V_i8, s_Q, s_K, s_V, B, H, Nq, Nk, d, causal, O, o_dtype, static_cast<float *>(ws),
                           static_cast<hipStream_t>(hip_stream));
}

