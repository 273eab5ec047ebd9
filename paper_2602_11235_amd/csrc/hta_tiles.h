// LDS tiles fed by asynchronous global -> LDS copies: offsets of MFMA operand fragments inside a swizzled tile, and
// the K/V stage of the row-stationary kernels.
//
// A tile is rows of D bf16, stored unpadded (row pitch D) with the XOR chunk swizzle of hta_mfma.h.  One wave-wide
// copy moves 1 KB: lane i lands at byte 16 i of the 1 KB block, i.e. at chunk position i % (D/8) of tile row
// (1 KB block index) * (64 / (D/8)) + i / (D/8); it therefore fetches the chunk that the swizzle assigns to that
// position.
#pragma once
#include "hta_mfma.h"

namespace hta {

// element offset, inside a swizzled tile, of the 16-byte fragment (row = lane % 32, chunk 2*ks + lane/32) that feeds
// an MFMA operand whose row index sits on the lane.  Adding a multiple of 32 rows leaves the swizzle unchanged.
template <int D>
__device__ inline void natural_offsets(int (&off)[D / 16], int lane) {
    const int l32 = lane & 31, hf = lane >> 5;
#pragma unroll
    for (int ks = 0; ks < D / 16; ks++) off[ks] = l32 * D + (((2 * ks + hf) ^ swizzle<D>(l32)) << 3);
}

// element offsets of the two 8-byte pieces of a transposed fragment: rows 4*hf + (lane%16)/4 and 8 below, 4 elements
// at column 32*db + 16*((lane/16)%2) + 4*(lane%4).  Adding a multiple of 16 rows leaves the swizzle unchanged.
template <int D>
__device__ inline void transposed_offsets(int (&lo)[D / 32], int (&hi)[D / 32], int lane) {
    const int pl = lane & 15, trow = 4 * (lane >> 5) + (pl >> 2);
#pragma unroll
    for (int db = 0; db < D / 32; db++) {
        const int chunk = 4 * db + 2 * ((lane >> 4) & 1) + ((pl & 3) >> 1);
        lo[db] = trow * D + ((chunk ^ swizzle<D>(trow)) << 3) + 4 * (pl & 1);
        hi[db] = (trow + 8) * D + ((chunk ^ swizzle<D>(trow + 8)) << 3) + 4 * (pl & 1);
    }
}

// K and V tiles of 64 keys each; one stage = [K tile][V tile].  The 2 * COPIES_PER_TILE copies of a stage are dealt
// to the NW waves of the workgroup, K copies first.
template <int D, int NW>
struct KvStage {
    static constexpr int BN = 64;
    static constexpr int TILE = BN * D;                       // elements
    static constexpr int BYTES = 2 * TILE * 2;                // K + V
    static constexpr int CPR = D / 8;                         // 16-byte chunks per row
    static constexpr int RPC = 64 / CPR;                      // rows per 1 KB copy
    static constexpr int COPIES_PER_TILE = BN / RPC;
    static constexpr int COPIES = 2 * COPIES_PER_TILE / NW;   // per wave and stage
    static_assert((2 * COPIES_PER_TILE) % NW == 0, "copies must split evenly over the waves");

    // loop-invariant byte offsets of the chunks this lane fetches, from the first element of (first key of the tile,
    // kv head g)
    __device__ static void lane_offsets(uint32_t (&voff)[COPIES], int Hkv, int wave, int lane) {
#pragma unroll
        for (int jj = 0; jj < COPIES; jj++) {
            const int j = (wave + jj * NW) % COPIES_PER_TILE;
            const int trow = j * RPC + lane / CPR;
            voff[jj] = (uint32_t)((trow * Hkv * D + (((lane % CPR) ^ swizzle<D>(trow)) << 3)) * 2);
        }
    }

    // Issue this wave's share of the copies of key tile t (keys 64 t .. 64 t + 63 of a history of length L) into the
    // stage at LDS byte address `stage`.  Keys past the history repeat key L-1: finite data whose weight the caller
    // forces to zero.  `wave_u` is the wave index as a uniform value.
    __device__ static void issue(const __bf16* kg, const __bf16* vg, int64_t kv_base, int Hkv, int g, int L, int t,
                                 uint32_t stage, const uint32_t (&voff)[COPIES], int wave_u, int lane) {
        const bool whole = (t + 1) * BN <= L;  // every key exists: no per-lane address arithmetic
        const int64_t tbase = ((kv_base + (int64_t)t * BN) * Hkv + g) * D;
#pragma unroll
        for (int jj = 0; jj < COPIES; jj++) {
            const int c = wave_u + jj * NW;
            const bool is_v = c >= COPIES_PER_TILE;
            const int j = is_v ? c - COPIES_PER_TILE : c;
            const uint32_t dst = stage + (is_v ? (uint32_t)TILE * 2u : 0u) + (uint32_t)j * 1024u;
            const __bf16* src = is_v ? vg : kg;
            if (whole) {
                copy16_global_to_lds_at(src + tbase, voff[jj], dst);
            } else {
                const int trow = j * RPC + lane / CPR;
                int key = t * BN + trow;
                key = key < L ? key : L - 1;
                const int chunk = (lane % CPR) ^ swizzle<D>(trow);
                copy16_global_to_lds_at(src + ((kv_base + key) * Hkv + g) * D + chunk * 8, dst);
            }
        }
    }
};

}  // namespace hta
