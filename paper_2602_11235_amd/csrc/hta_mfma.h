// gfx950 device helpers shared by the bf16 MFMA kernels: vector types, the 32x32x16 bf16 MFMA,
// the LDS transpose read, cross-half exchanges.
//
// Lane layouts (wave of 64 lanes, lane = 32*hf + l32; checked on hardware):
//   v_mfma_f32_32x32x16_bf16  D[32x32] += A[32x16] B[16x32]
//     A operand: lane holds row m = l32, the 8 consecutive k values 8*hf .. 8*hf+7
//     B operand: lane holds column n = l32, the 8 consecutive k values 8*hf .. 8*hf+7
//     D (16 floats): lane holds column n = l32, register v holds row m = 8*(v/4) + 4*hf + (v%4)
//   Because the contraction index of the accumulator's *registers* is m, an accumulator can be fed
//   back (after conversion to bf16) as the B operand of a product that contracts over m: registers
//   8*s .. 8*s+7 become k-step s, whose k-slot j of half hf is row m = 16*s + 8*(j/4) + 4*hf + (j%4).
//   ds_read_b64_tr_b16: inside each group of 16 lanes, lane i receives element (i%4) of the four
//     8-byte chunks addressed by lanes (i/4), (i/4)+4, (i/4)+8, (i/4)+12 of the group.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace hta {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

#define HTA_LDS __attribute__((address_space(3)))

// f(integral_constant<int, I>) for I = 0 .. N-1, unrolled at compile time (keeps register arrays out of scratch)
template <int I, int N, typename F>
__device__ inline void static_for(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

__device__ inline floatx16 mfma32(bf16x8 a, bf16x8 b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Pointwise weights (the SiLU reading of phi2) for a raw dot product s, x = scale s:
//   sigma = 1 / (1 + 2^(-x log2 e)),  silu(x) = x sigma,  silu'(x) = sigma (1 + x (1 - sigma)).
// neg_c2 = -scale log2(e).  A masked entry carries s = -1e30 (finite on purpose): then sigma is exactly 0 and both
// results are zero, where -inf would give inf * 0.
constexpr float PW_MASKED = -1e30f;
__device__ inline float pw_sigmoid(float s, float neg_c2) { return __builtin_amdgcn_rcpf(1.f + fast_exp2(s * neg_c2)); }
__device__ inline float pw_silu(float x, float sg) { return x * sg; }
__device__ inline float pw_silu_prime(float x, float sg) { return fmaf(sg, x * (1.f - sg), sg); }
// the same from silu(x) = x sigma, where that is at hand: silu'(x) = sigma + silu(x) (1 - sigma)
__device__ inline float pw_silu_prime_of(float silu, float sg) { return fmaf(silu, 1.f - sg, sg); }

// value held by the lane 32 positions away (the other half of the wave); v_permlane32_swap is a VALU
// exchange of the upper half of its first operand with the lower half of its second
__device__ inline float other_half(float x) {
    const unsigned u = __builtin_bit_cast(unsigned, x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    // lanes 0..31 now hold (own, upper partner), lanes 32..63 hold (lower partner, own)
    return __builtin_bit_cast(float, (threadIdx.x & 32) ? r[0] : r[1]);
}

// acc + x[0] + x[1] + ... + x[7] for eight packed bf16 values (v_dot2c_f32_bf16 against packed ones), two chains
__device__ inline void add_bf16x8(float& acc0, float& acc1, bf16x8 x) {
    bf16x2 one;
    one[0] = (__bf16)1.0f;
    one[1] = (__bf16)1.0f;
    const bf16x2 a = __builtin_shufflevector(x, x, 0, 1), b = __builtin_shufflevector(x, x, 2, 3);
    const bf16x2 c = __builtin_shufflevector(x, x, 4, 5), d = __builtin_shufflevector(x, x, 6, 7);
    acc0 = __builtin_amdgcn_fdot2_f32_bf16(a, one, acc0, false);
    acc1 = __builtin_amdgcn_fdot2_f32_bf16(b, one, acc1, false);
    acc0 = __builtin_amdgcn_fdot2_f32_bf16(c, one, acc0, false);
    acc1 = __builtin_amdgcn_fdot2_f32_bf16(d, one, acc1, false);
}

// acc + <x, y> for eight packed bf16 pairs: products are exact in float32, sums are float32
__device__ inline float dot_bf16x8(float acc, bf16x8 x, bf16x8 y) {
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(x, x, 0, 1), __builtin_shufflevector(y, y, 0, 1), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(x, x, 2, 3), __builtin_shufflevector(y, y, 2, 3), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(x, x, 4, 5), __builtin_shufflevector(y, y, 4, 5), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(x, x, 6, 7), __builtin_shufflevector(y, y, 6, 7), acc, false);
    return acc;
}

// wait until every outstanding vector-memory load of this wave has landed
__device__ inline void wait_vmem_loads() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// Transposed 8-key fragment out of a row-major [row][col] bf16 tile in LDS.
// The calling lane receives, for column `col0 + (lane%16)` of its 16-lane group, the elements of rows
// row0 .. row0+3 (first read) and row0+8 .. row0+11 (second read).  `tile` points at element (0,0),
// `stride` is the row pitch in elements; row0 / col0 must be uniform per 16-lane group, col0 % 4 == 0.
__device__ inline bf16x8 lds_read_tr_8(const __bf16* tile, int stride, int row0, int col0, int lane) {
    const int p = lane & 15;
    const __bf16* a0 = tile + (row0 + (p >> 2)) * stride + col0 + 4 * (p & 3);
    const __bf16* a1 = a0 + 8 * stride;
    short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((HTA_LDS short4v*)(HTA_LDS char*)a0);
    short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((HTA_LDS short4v*)(HTA_LDS char*)a1);
    typedef short short8v __attribute__((ext_vector_type(8)));
    short8v r = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, r);
}

// The two 8-byte transposed reads of lds_read_tr_8 at precomputed per-lane addresses (rows r..r+3 and r+8..r+11).
__device__ inline bf16x8 lds_read_tr_pair(const __bf16* a0, const __bf16* a1) {
    short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((HTA_LDS short4v*)(HTA_LDS char*)a0);
    short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((HTA_LDS short4v*)(HTA_LDS char*)a1);
    typedef short short8v __attribute__((ext_vector_type(8)));
    short8v r = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, r);
}

// Unpadded LDS tiles (row pitch = D elements) with an XOR swizzle of their 16-byte chunks: the chunk that holds
// elements 8c .. 8c+7 of row `row` sits at chunk position c ^ swizzle<D>(row).  Chosen so that both access
// patterns of the kernels are free of bank conflicts: 16 lanes reading the same chunk of 16 consecutive rows,
// and 32 lanes reading four consecutive chunks of four consecutive rows (the transposed read).
template <int D>
__device__ inline int swizzle(int row) {
    if (D == 32) return (row >> 2) & 3;
    if (D == 64) return (((row >> 1) & 1) << 2) | ((row >> 2) & 3);
    return ((row & 3) << 2) | ((row >> 2) & 3);
}

// Asynchronous 16-byte copy global -> LDS without a register stop-over: lane i of the wave writes
// lds_wave_base[16 i .. 16 i + 15] with the 16 bytes at its own global address (lds_wave_base must be the same
// for all lanes).  Completion is tracked by the wave's vector-memory counter like any load, and is the caller's
// business (wait_vmem_outstanding): the copy is issued from inline assembly precisely so that the compiler does
// not drain it before every later LDS read.  The statement overwrites M0 and says so in its clobber list:
// the compiler reserves M0 for itself and sets it right before each use of its own, but its pass that merges equal M0
// initialisations has to see that one was destroyed in between.  Its own vmcnt waits for ordinary loads ignore these copies, which
// only makes them wait longer than needed, never less (the counter retires in issue order).
__device__ inline void copy16_global_to_lds(const void* global_lane_ptr, void* lds_wave_base) {
    const uint32_t base =
        __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)lds_wave_base);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(base), "v"(global_lane_ptr) : "memory", "m0");
}

// Same for 4 bytes per lane: lane i writes lds_wave_base[4 i .. 4 i + 3].
__device__ inline void copy4_global_to_lds(const void* global_lane_ptr, void* lds_wave_base) {
    const uint32_t base =
        __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)lds_wave_base);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off" : : "s"(base), "v"(global_lane_ptr) : "memory", "m0");
}

// The same copies with the LDS destination given as a byte address inside LDS (wave-uniform), which spares the
// address-space conversion of a generic pointer; lds_address() of a pointer into a __shared__ array is that address.
__device__ inline uint32_t lds_address(const void* p) { return (uint32_t)(uintptr_t)(HTA_LDS const void*)p; }

__device__ inline void copy16_global_to_lds_at(const void* global_lane_ptr, uint32_t lds_wave_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(lds_wave_addr), "v"(global_lane_ptr) : "memory", "m0");
}

__device__ inline void copy4_global_to_lds_at(const void* global_lane_ptr, uint32_t lds_wave_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off" : : "s"(lds_wave_addr), "v"(global_lane_ptr) : "memory", "m0");
}

// 16-byte copy whose global address is a wave-uniform base plus a per-lane unsigned byte offset: no address
// arithmetic on the vector unit at all when the per-lane offsets are loop-invariant.
__device__ inline void copy16_global_to_lds_at(const void* uniform_base, uint32_t lane_byte_offset, uint32_t lds_wave_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(lds_wave_addr), "v"(lane_byte_offset), "s"(uniform_base) : "memory", "m0");
}

// wait until at most N vector-memory operations of this wave are still outstanding (N < 64)
template <int N>
__device__ inline void wait_vmem_outstanding() {
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | 0x0F70);
}

// all LDS traffic of this wave has completed, then wait for the other waves of the workgroup: orders LDS stores
// and loads across the workgroup without also waiting for global loads that are still in flight
__device__ inline void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

}  // namespace hta
