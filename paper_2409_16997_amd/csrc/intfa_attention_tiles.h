// K / V tile layout in LDS, MFMA operand addressing and the direct-to-LDS staging copies shared by the attention
// kernels of intfa_attention.hip (the fused kernel) and intfa_attention_fewq.hip (few queries per head).
#ifndef INTFA_ATTENTION_TILES_H
#define INTFA_ATTENTION_TILES_H

#include "intfa_device.h"

namespace ifa_tiles {

using namespace ifa_dev;

constexpr int BC = 128;       // keys per block: the B_c of Algorithm 1
constexpr float LOG2_R_NORM = -9.01129329928057f;   // log2(127 / 65535): P / 65535 is what the 16-bit normalised conversion takes

// Slot swizzles.  Logical 16-byte chunk c of row `row` is stored in slot c ^ swz(row).
// K is read with ds_read_b128 by 32 consecutive rows at one chunk: 8 consecutive rows must fall in 8
// different slots of a 128-byte line.  V is read with ds_read_b64_tr_b8, where a 16-lane group touches
// rows {0-3, 8-11} or {4-7, 12-15} (mod 16) of a tile at one chunk: bits 0, 1 and 3 of the row
// separate those 8 rows.
template <int D> __device__ __forceinline__ int k_swz(int row) {
    return (D == 128) ? (row & 7) : ((row >> 1) & 3);
}
template <int D> __device__ __forceinline__ int v_swz(int row) {
    const int s = (row & 3) | ((row >> 1) & 4);
    return (D == 128) ? s : (s & 3);
}

#if defined(__HIP_DEVICE_COMPILE__)   // device-only code: buffer resources and LDS builtins do not exist in the host pass
// Per-lane LDS byte offsets of the MFMA operands inside a K / V tile (tile- and block-independent).
template <int D> struct LaneOffsets {
    // A operand of S^T = K Q^T, k-step kk: row r, chunk 2*kk + g.  The swizzle is an XOR on the chunk index and
    // 2*kk + g = 2*kk ^ g, so the offset of step kk is k0 ^ (32*kk): one register serves all steps (+ 32*mt*D per
    // key tile, an immediate).
    unsigned k0;
    // A operand of O^T = V^T P^T, d tile dt, bytes 0..7 of the operand: v0 ^ (32*dt) by the same argument; bytes
    // 8..15 come from the key 16 rows further on, which the swizzle does not see: + 16*D (+ 32*mt*D per key tile).
    unsigned v0;
    int sk;               // first of this lane's s_K values in a 32-key tile (+ 128*mt + 32*vq bytes)
    // staging: byte offset inside the K / V tile in HBM of the chunk this lane moves in piece i of its wavefront.
    // Piece i covers rows 1024 i / D further on, and the row bits the swizzles look at do not change with i except
    // one bit of the V swizzle (D = 128) that follows the parity of i: offset(i) = gk + 1024 i for K and
    // gv[i & 1] + 1024 (i - (i & 1)) for V, the multiples of 1024 going into the scalar offset of the copy.
    unsigned gk;
    unsigned gv[2];
    __device__ __forceinline__ LaneOffsets(int lane, int wave) {
        const int r = lane & 31, g = lane >> 5;
        constexpr int CH = D / 16, ITER = D / 32;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int p = (wave * ITER + i) * 64 + lane, row = p / CH, slot = p % CH;
            if (i == 0) gk = row * D + 16 * (slot ^ k_swz<D>(row));
            gv[i] = row * D + 16 * (slot ^ v_swz<D>(row));
        }
        k0 = r * D + ((g ^ k_swz<D>(r)) * 16);
        // transposing read: 16-lane group G = lane / 16 serves d columns 16*(G%2) .. +15 of the tile and key
        // half g = G / 2; lane i of the group addresses row (i / 2) of its 8 keys, byte half (i % 2).
        const int i = lane & 15, G = lane >> 4, kidx = i >> 1, par = i & 1;
        const int key = 8 * (kidx >> 2) + 4 * g + (kidx & 3);        // accumulator row order
        v0 = key * D + (((G & 1) ^ v_swz<D>(key)) * 16) + 8 * par;
        sk = 16 * g;
    }
};

template <int D> __device__ __forceinline__ lds_ptr k_operand(lds_ptr ks, const LaneOffsets<D> &lo, int kk) {
    return lds_xor(ks, 32 * kk, lo.k0);
}
template <int D> __device__ __forceinline__ lds_ptr v_operand(lds_ptr vs, const LaneOffsets<D> &lo, int dt) {
    return lds_xor(vs, 32 * dt, lo.v0);
}

// What the next key block needs staged.  The copies are buffer_load_dwordx4 ... lds: the tensor's base and
// size sit in a scalar buffer resource, the block offset in a scalar register and the lane's chunk offset in
// one loop-invariant VGPR, so a copy costs no vector ALU work, and reads past the tensor return zero instead
// of faulting.  One "piece" is one such instruction of this wavefront (1 KB); a wavefront moves D/32 pieces of
// K and of V per block, issued one pair at a time between the MFMA groups of S^T so that the four wavefronts
// of a workgroup do not all queue on the vector-memory port at once and every copy has the rest of the block
// to land.
//
// The copies are written as inline assembly on purpose.  Issued through the compiler's builtin they count as
// stores to LDS that any later transposing LDS read might alias, and the compiler then waits for ALL of them
// (vmcnt(0)) in front of the first V^T operand read of the block, which exposes the HBM latency in the middle
// of every block.  They cannot alias: the copies fill the other half of the double buffer, and the wait that
// does order them (wait_all_memory + barrier at the end of the block) is explicit.  M0 holds the LDS
// destination of such a copy; nothing else in this kernel uses M0.
struct Prefetch {
    BufRsrc k, v, sk;                // one head's K [N, d], V [N, d] int8 and s_K [N] fp32
    int koff, skoff;                 // byte offset of the next block inside K (= inside V) and inside s_K
    lds_ptr lk, lv, lsk;             // LDS destinations (tile bases)
};
// Block offset of a request that must fetch nothing (no block follows): past the end of any tensor, so that every
// lane is out of range -- the scalar offset takes part in the range check (probed on this chip) -- and nothing is
// read from memory.  The LDS destination IS still written (with zeros), so it must be a buffer nobody uses until the
// next wait + barrier.  Cheaper than a branch around each copy: the block stays one basic block for the scheduler.
constexpr int NOWHERE = 0x7fff0000;

// (NT: with the non-temporal hint, for the passes that read every byte once)
template <int D, bool NT = false>
__device__ __forceinline__ void prefetch_k_piece(const Prefetch &nx, const LaneOffsets<D> &lo, int wave, int i) {
    if (NT) lds_copy16_nt(nx.k, nx.lk + (wave * (D / 32) + i) * 1024, lo.gk, nx.koff + 1024 * i);
    else lds_copy16(nx.k, nx.lk + (wave * (D / 32) + i) * 1024, lo.gk, nx.koff + 1024 * i);
}
template <int D, bool NT = false>
__device__ __forceinline__ void prefetch_v_piece(const Prefetch &nx, const LaneOffsets<D> &lo, int wave, int i) {
    if (NT) lds_copy16_nt(nx.v, nx.lv + (wave * (D / 32) + i) * 1024, lo.gv[i & 1], nx.koff + 1024 * (i - (i & 1)));
    else lds_copy16(nx.v, nx.lv + (wave * (D / 32) + i) * 1024, lo.gv[i & 1], nx.koff + 1024 * (i - (i & 1)));
}
__device__ __forceinline__ void prefetch_sk(const Prefetch &nx, int wave, int lane) {
    // 2 x 64 lanes x 4 bytes = the 128 scales of the block, by wavefronts 2 and 3.  Dword copies: a head's
    // scales start at an arbitrary 4-byte boundary when N is not a multiple of 4.
    if (wave >= 2) lds_copy4(nx.sk, nx.lsk + 256 * (wave - 2), 4 * lane + 256 * (wave - 2), nx.skoff);
}


// s_waitcnt that waits only for the vector-memory counter to drop to n (gfx9 encoding: vmcnt in bits 3:0 and 15:14)
template <int N> __device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}
#endif  // __HIP_DEVICE_COMPILE__

}  // namespace ifa_tiles

#endif
