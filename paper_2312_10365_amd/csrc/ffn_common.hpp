// Device-side building blocks shared by the routed-FFN GEMM kernels (gfx950 only): the LDS DMA
// copy, the hand-placed wait, LDS slot swizzles, the transposing LDS read, the MFMA row
// permutation, and the row-tile record of the schedule tables.
#pragma once
#include "spt_device.hpp"

namespace spt {

constexpr int TILE = 128;  // output tile edge of the narrow-block kernels

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ bf16x8 as_bf16x8(const uint4& v) { return __builtin_bit_cast(bf16x8, v); }

// "Fragment order" of the per-pair hidden values of narrow blocks (act(H), dHpre: written by the
// K = d GEMM, read by the K = Bs and the weight-gradient GEMMs): 32 consecutive sorted positions x
// 16 consecutive hidden units form one contiguous kilobyte, [position / 32][unit / 16]
// [position % 32][unit % 16].  A wavefront whose lanes hold consecutive positions then reads one
// K-step of a 32-row MFMA operand as one contiguous kilobyte instead of 32 pieces 2 Bs bytes
// apart.  A tensor of P positions holds ceil(P / 32) * 32 rows.
__host__ __device__ __forceinline__ size_t hfrag_off(int q, int u, int Bs) {
  return ((size_t)(q >> 5) * (size_t)(Bs >> 4) + (size_t)(u >> 4)) * 512 + (size_t)((q & 31) * 16 + (u & 15));
}
template <bool FRAG>
__device__ __forceinline__ size_t hval_off(int q, int u, int Bs) {
  return FRAG ? hfrag_off(q, u, Bs) : (size_t)q * Bs + u;
}

// One row tile of a bucket in an XCD's run order: bucket id and first sorted position.
struct KdTile { int32_t bucket, q0; };

// 16-byte slot of (row, chunk) in a stage region with 4 chunks (64 bytes, 32 K-values) per row.
__device__ __forceinline__ int kd_slot(int row, int chunk) { return row * 4 + (chunk ^ ((row >> 2) & 3)); }

// Asynchronous copy global -> LDS, 16 bytes per lane; lane L's data lands at lds_base + 16 L.
__device__ __forceinline__ void dma16(const void* gptr, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(gptr) : "memory");
}
// s_waitcnt vmcnt(N) alone (N <= 63): the other counters are left at their maxima.
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0xF << 8));
}

// Between a wavefront's LDS writes and its own reads of what OTHER lanes wrote (and before it
// overwrites what they read): LDS executes one wavefront's accesses in order, so no wait is
// needed; this keeps the compiler from moving the accesses across each other.
__device__ __forceinline__ void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// MFMA row i of a 32-row tile can be fed any operand row; feeding it row
// rho32(i) = 16*((i>>2)&1) + 4*(i>>3) + (i&3) makes the 16 accumulator values of a lane 16
// CONSECUTIVE rows of the operand.
__device__ __forceinline__ int rho32(int i) { return 16 * ((i >> 2) & 1) + 4 * (i >> 3) + (i & 3); }

// ds_read_b64_tr_b16 hands each lane 4 consecutive K-values of ONE column out of a K-major
// tile.  Within a group of 16 lanes, lane s points at row (s >> 2), 4-column group (s & 3), and
// result[j][e] = memory[address of lane 4e + (j >> 2)][j & 3].  Two of them make one 8-value
// MFMA operand fragment.
typedef short v4s __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) v4s* lds_v4s_ptr;

__device__ __forceinline__ bf16x8 tr_read_frag(const char* lds_lo, const char* lds_hi) {
  struct { v4s a, b; } t;
  t.a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)(uintptr_t)lds_lo);
  t.b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)(uintptr_t)lds_hi);
  return __builtin_bit_cast(bf16x8, t);
}

}  // namespace spt
