// K = Bs contraction of the routed FFN for blocks of at most 128 hidden units, with the
// write-back of Algorithm 4 (line 5, block outputs ADDED per token) folded into the GEMM:
//
//   out[t][:] = sum over the blocks b that token t activates, ascending b, of
//               Hin[position of (t, b)][:] * W[b]            (+ Z[t][:], the low-rank term)
//
// forward: Hin = act(H), W = W2, out = Y;  backward: Hin = dHpre, W = W1, out = dX.
//
// The GEMM is token-range stationary.  A workgroup owns R consecutive tokens x C output columns
// as an fp32 slab in LDS and walks the N blocks in order.  Inside a bucket the sorted positions
// ascend with the token id, so the rows of block b that belong to the workgroup's tokens are one
// contiguous run [rstart[r][b], rstart[r+1][b]) -- about R k / N of them.  The run is multiplied
// by the block's C weight columns on the matrix cores (v_mfma_f32_32x32x16_bf16; bucket rows on
// the lane axis, output columns on the register axis, permuted by rho32 so a lane holds 16
// consecutive columns of ITS row) and every lane adds its 64 bytes into the LDS row of its
// token.  A token occurs at most once per block, the blocks come in ascending order and a
// barrier separates them, so every output element is summed in fp32 in one fixed order -- no
// atomics, no partial rows in HBM, one rounding to bf16 when the slab is written out.
//
// Operands.  The weight slice (Bs x C, hidden-unit major as stored) is copied into a single LDS
// stage by global_load_lds_dwordx4 and turned into K-contiguous MFMA fragments by
// ds_read_b64_tr_b16; the fragments of a block live in registers, so the stage is free for the
// next block's copy as soon as they are read.  Rows of Hin are K-contiguous in memory and go
// straight from global memory into the lane that owns the row (16 bytes per K-step), one block
// ahead of their use.  Four wavefronts: (row tile rw, column half cw); a run longer than 64 rows
// takes more passes over the same register-resident weight fragments.
//
// LDS slab rows are padded by 16 bytes: the 16-byte accesses of a lane group then spread over
// the banks by token id (measured 65 % of the LDS peak with random rows, against 100 % for
// consecutive rows and 30 % for 4-byte accesses with the lanes on the column axis; the LDS
// float atomic add runs at a hundredth of that rate).
#include <stdlib.h>
#include <type_traits>

#include "ffn_common.hpp"
#include "spt_host.hpp"
#include "profile.hpp"

namespace spt {

constexpr int SC_CC = 64;          // output columns per weight chunk (128-byte LDS rows)
constexpr int SC_PAD = 16;         // bytes of padding per slab row
constexpr int SC_THREADS = 256;

__device__ __forceinline__ void sc_wait_all() { __builtin_amdgcn_s_waitcnt(0); }
__device__ __forceinline__ void sc_wait_lds() { __builtin_amdgcn_s_waitcnt(0xC07F); }  // lgkmcnt(0) only
__device__ __forceinline__ void sc_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

// rstart[r][b] = first sorted position of bucket b whose token id is >= r * R (r = 0 .. nr):
// a lower bound on perm, whose entries t * k + j ascend inside a bucket.
__global__ __launch_bounds__(256) void scatter_ranges_kernel(const int32_t* __restrict__ offsets,
                                                             const int32_t* __restrict__ perm, int N,
                                                             int k, int R, int nr,
                                                             int32_t* __restrict__ rstart) {
  const int id = blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= (nr + 1) * N) return;
  const int r = id / N, b = id % N;
  int lo = offsets[b], hi = offsets[b + 1];
  const int64_t key = (int64_t)r * R * k;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if ((int64_t)perm[mid] < key) lo = mid + 1; else hi = mid;
  }
  rstart[id] = lo;
}

// KS = Bs / 16 K-steps per block.  A workgroup owns R tokens x 64 output columns; wavefront w
// owns row tile w (32 bucket rows) of every pass over a run and both 32-column tiles.
constexpr int SC_C = 64;                     // output columns per workgroup
constexpr int SC_STRIDE = SC_C * 4 + SC_PAD; // bytes per slab row
constexpr int SC_STAGES = 3;                 // weight-slice ring: two copies in flight

template <int KS>
__global__ __launch_bounds__(SC_THREADS, 1) void ffn_scatter_kernel(
    const uint16_t* __restrict__ Hin, const uint16_t* __restrict__ W,
    const int32_t* __restrict__ rstart, const int32_t* __restrict__ tok, int N, int d, int T, int R,
    int nr, int nslab, uint16_t* __restrict__ out, const uint16_t* __restrict__ Z) {
  constexpr int Bs = KS * 16;
  constexpr int NW = KS / 2;                   // weight-copy instructions per wavefront and block
  constexpr int STAGE_BYTES = Bs * 128;
  constexpr int GROUP = NW + KS + 1;           // vector-memory instructions per prefetched block
  extern __shared__ uint4 sc_smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int i = lane & 31, h = lane >> 5;

  // Work item.  With a multiple of 8 slabs an XCD (workgroup id mod 8) keeps to its own slabs
  // and the workgroups it runs together are token ranges x up to 4 slabs: per block they want
  // a few weight slices and a few runs of Hin rows, which its L2 serves to all of them.
  int r, slab;
  if (nslab % 8 == 0) {
    const int spx = nslab >> 3, x = blockIdx.x & 7, j = blockIdx.x >> 3;
    const int inner = spx < 4 ? spx : 4;       // slabs that run side by side
    const int grp = j / (inner * nr), rem = j % (inner * nr);
    slab = x * spx + grp * inner + rem % inner;
    r = rem / inner;
    if (grp * inner + rem % inner >= spx) return;
  } else {
    slab = blockIdx.x % nslab;
    r = blockIdx.x / nslab;
  }
  if (r >= nr) return;
  const int t0 = r * R, c0 = slab * SC_C;
  const int rows = (T - t0 < R) ? T - t0 : R;

  char* slab_lds = reinterpret_cast<char*>(sc_smem);
  const uint32_t ring_lds = (uint32_t)(uintptr_t)sc_smem + (uint32_t)(R * SC_STRIDE);
  const char* ring = slab_lds + R * SC_STRIDE;

  for (int o = tid * 16; o < R * SC_STRIDE; o += SC_THREADS * 16)
    *reinterpret_cast<uint4*>(slab_lds + o) = make_uint4(0u, 0u, 0u, 0u);

  typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;
  const const_i32_ptr rs0 = (const_i32_ptr)(uintptr_t)(rstart + (size_t)r * N);
  const const_i32_ptr rs1 = (const_i32_ptr)(uintptr_t)(rstart + (size_t)(r + 1) * N);
  struct Run { int b, lo, hi; };
  auto next_run = [&](int after) {  // next block with rows for these tokens (wave-uniform scalar loads)
    Run x{after + 1, 0, 0};
    for (; x.b < N; ++x.b) { x.lo = rs0[x.b]; x.hi = rs1[x.b]; if (x.hi > x.lo) break; }
    return x;
  };

  // weight copy: instruction j of this wavefront fills stage rows 8 (wave NW + j) .. + 7 (a stage
  // row = 128 bytes = one hidden unit x 64 columns); lane L -> row + L / 8, physical 16-byte slot
  // L % 8 = logical ^ (((row >> 1) & 1) << 2)
  int w_off[NW];
#pragma unroll
  for (int j = 0; j < NW; ++j) {
    const int unit = 8 * (wave * NW + j) + (lane >> 3);
    const int ch = (lane & 7) ^ (((unit >> 1) & 1) << 2);
    w_off[j] = unit * d + c0 + ch * 8;
  }
  auto issue_w = [&](int b, int stage) {
    const uint16_t* wb = W + (size_t)b * Bs * d;
#pragma unroll
    for (int j = 0; j < NW; ++j)
      dma16(wb + w_off[j],
            __builtin_amdgcn_readfirstlane(ring_lds + (uint32_t)(stage * STAGE_BYTES + (wave * NW + j) * 1024)));
  };

  // transposing fragment reads (natural K order: lane half h holds units 16 s + 8 h .. + 7):
  // lane (g = lane / 16, sl = lane % 16) points at stage row 16 s + 8 (g >> 1) + 4 rr + (sl >> 2)
  // and at the 4-column group that gives MFMA row 16 (g & 1) + j the output column rho32 of it.
  const int g = lane >> 4, sl = lane & 15, a4 = sl & 3;
  const int colgrp = 4 * (a4 & 1) + 2 * (g & 1) + (a4 >> 1);
  uint32_t tr_off[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const int krow = 8 * (g >> 1) + (sl >> 2);
    const int col = t * 32 + 4 * colgrp;
    const int ch = (col >> 3) ^ (((krow >> 1) & 1) << 2);
    tr_off[t] = (uint32_t)(krow * 128 + ch * 16 + (col & 4) * 2);
  }

  // Hin rows of (run, row tile): 16 bytes per K-step for the lane's row; lanes past the run's
  // end read its first row and add nothing.  The prefetching loads are written as asm so that the
  // compiler's own vmcnt bookkeeping never sees them (it would otherwise wait for the youngest
  // load whenever control flow merges): the loop waits with constants and then "pins" the
  // registers, which orders every use behind the wait.
  struct RowTile { bf16x8 hb[KS]; int tokv; bool live; };
  auto row_of = [&](RowTile& rt, const Run& run, int tile) {
    const int q = run.lo + tile * 32 + i;
    rt.live = q < run.hi;
    return rt.live ? q : run.lo;
  };
  auto prefetch_rows = [&](RowTile& rt, const Run& run, int tile) {
    const int qq = row_of(rt, run, tile);
    const int32_t* tp = tok + qq;
    const uint16_t* src = Hin + (size_t)qq * Bs + 8 * h;
    asm volatile("global_load_dword %0, %1, off" : "=v"(rt.tokv) : "v"(tp) : "memory");
#pragma unroll
    for (int s = 0; s < KS; ++s)
      asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(rt.hb[s]) : "v"(src + 16 * s) : "memory");
  };
  auto pin_rows = [&](RowTile& rt) {
    asm volatile("" : "+v"(rt.tokv));
#pragma unroll
    for (int s = 0; s < KS; ++s) asm volatile("" : "+v"(rt.hb[s]));
  };
  auto load_rows = [&](RowTile& rt, const Run& run, int tile) {
    const int qq = row_of(rt, run, tile);
    rt.tokv = tok[qq];
    const uint4* src = reinterpret_cast<const uint4*>(Hin + (size_t)qq * Bs + 8 * h);
#pragma unroll
    for (int s = 0; s < KS; ++s) rt.hb[s] = as_bf16x8(src[2 * s]);
  };

  bf16x8 af[2][KS];
  auto multiply_add = [&](const RowTile& rt) {
    f32x16 acc[2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int s = 0; s < KS; ++s)
        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[t][s], rt.hb[s], acc[t], 0, 0, 0);
    if (rt.live) {
      char* rowp = slab_lds + (rt.tokv - t0) * SC_STRIDE + 64 * h;
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        f32x4* p = reinterpret_cast<f32x4*>(rowp + t * 128);
        f32x4 v0 = p[0], v1 = p[1], v2 = p[2], v3 = p[3];
        const f32x16& c = acc[t];
        v0 += f32x4{c[0], c[1], c[2], c[3]};
        v1 += f32x4{c[4], c[5], c[6], c[7]};
        v2 += f32x4{c[8], c[9], c[10], c[11]};
        v3 += f32x4{c[12], c[13], c[14], c[15]};
        p[0] = v0; p[1] = v1; p[2] = v2; p[3] = v3;
      }
    }
  };

  // Prefetch two runs ahead: the weight slice into the ring, the first pass's Hin rows into
  // registers.  Every prefetched run costs GROUP vector-memory instructions per wavefront, so
  // "the current run has landed" is a constant vmcnt wait.  The loop is unrolled by the ring
  // depth: stage and register buffer of a run are compile-time constants, so no prefetched
  // register is ever copied (a copy would have to wait for the load that fills it).
  Run r0 = next_run(-1), r1 = next_run(r0.b), r2 = next_run(r1.b);
  RowTile hbuf[SC_STAGES];
  if (r0.b < N) { issue_w(r0.b, 0); prefetch_rows(hbuf[0], r0, wave); }
  if (r1.b < N) { issue_w(r1.b, 1); prefetch_rows(hbuf[1], r1, wave); }
  auto iteration = [&](auto cur_tag) {
    constexpr int cur = decltype(cur_tag)::value;
    constexpr int fill = (cur + 2) % SC_STAGES;
    // own copies and rows of this run have landed (the next run's GROUP may be in flight)
    if (r1.b < N) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(GROUP) : "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    pin_rows(hbuf[cur]);
    sc_wait_lds();                                            // own slab updates of the last run are done
    sc_barrier();                                             // ... and everyone's
    if (r2.b < N) {
      issue_w(r2.b, fill);
      prefetch_rows(hbuf[fill], r2, wave);
    }
    const char* st = ring + cur * STAGE_BYTES;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int s = 0; s < KS; ++s)
        af[t][s] = tr_read_frag(st + tr_off[t] + s * 2048, st + tr_off[t] + s * 2048 + 512);
    multiply_add(hbuf[cur]);
    for (int tile = 4 + wave; tile * 32 < r0.hi - r0.lo; tile += 4) {
      RowTile extra;
      load_rows(extra, r0, tile);
      multiply_add(extra);
    }
    r0 = r1; r1 = r2; r2 = next_run(r2.b < N ? r2.b : N - 1);
  };
  while (true) {
    if (r0.b >= N) break;
    iteration(std::integral_constant<int, 0>{});
    if (r0.b >= N) break;
    iteration(std::integral_constant<int, 1>{});
    if (r0.b >= N) break;
    iteration(std::integral_constant<int, 2>{});
  }
  sc_wait_all();
  sc_barrier();

  // write the slab out: one rounding to bf16 (+ the low-rank row of the token, if any)
  constexpr int CG = SC_C / 8;  // 16-byte output pieces per row
  for (int it = tid; it < rows * CG; it += SC_THREADS) {
    const int row = it / CG, cg = it % CG;
    const f32x4* p = reinterpret_cast<const f32x4*>(slab_lds + row * SC_STRIDE + cg * 32);
    f32x4 lo4 = p[0], hi4 = p[1];
    const size_t o = (size_t)(t0 + row) * d + c0 + cg * 8;
    if (Z) {
      const uint4 z = *reinterpret_cast<const uint4*>(Z + o);
      lo4 += f32x4{lo_bf16(z.x), hi_bf16(z.x), lo_bf16(z.y), hi_bf16(z.y)};
      hi4 += f32x4{lo_bf16(z.z), hi_bf16(z.z), lo_bf16(z.w), hi_bf16(z.w)};
    }
    *reinterpret_cast<uint4*>(out + o) =
        make_uint4(pack_bf16x2(lo4[0], lo4[1]), pack_bf16x2(lo4[2], lo4[3]), pack_bf16x2(hi4[0], hi4[1]),
                   pack_bf16x2(hi4[2], hi4[3]));
  }
}

// ------------------------------------------------------------------------------------------
// host side
ScatterPlan plan_scatter(const spt_shape_t& s) {
  ScatterPlan p;
  const int budget = 160 * 1024 - SC_STAGES * s.Bs * 128;
  int rmax = budget / SC_STRIDE;
  if (rmax > 448) rmax = 448;
  if (const char* e = getenv("SPT_SC_R")) { const int v = atoi(e); if (v >= 8 && v <= budget / SC_STRIDE) rmax = v; }
  p.nslab = s.d / SC_C;
  // ranges: as few as the LDS slab allows, but enough workgroups to occupy the chip when the
  // shape is small (never below 64 tokens per range)
  p.nr = (s.T + rmax - 1) / rmax;
  const int fill = (256 + p.nslab - 1) / p.nslab, cap = (s.T + 63) / 64;
  if (p.nr < fill) p.nr = fill < cap ? fill : (cap > p.nr ? cap : p.nr);
  p.R = (s.T + p.nr - 1) / p.nr;
  p.nr = (s.T + p.R - 1) / p.R;
  p.smem = p.R * SC_STRIDE + SC_STAGES * s.Bs * 128;
  p.table_bytes = align256((size_t)(p.nr + 1) * s.N * 4);
  return p;
}

hipError_t run_scatter_ranges(const spt_shape_t& s, const ScatterPlan& p, const int32_t* offsets,
                              const int32_t* perm, int32_t* rstart, hipStream_t st) {
  const int n = (p.nr + 1) * s.N;
  scatter_ranges_kernel<<<(n + 255) / 256, 256, 0, st>>>(offsets, perm, s.N, s.k, p.R, p.nr, rstart);
  return hipGetLastError();
}

template <int KS>
static hipError_t launch_scatter_t(const spt_shape_t& s, const ScatterPlan& p, const uint16_t* Hin,
                                   const uint16_t* W, const int32_t* rstart, const int32_t* tok,
                                   uint16_t* out, const uint16_t* Z, hipStream_t st) {
  static bool attr_set = false;
  if (!attr_set) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(ffn_scatter_kernel<KS>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  int grid;
  if (p.nslab % 8 == 0) {
    const int spx = p.nslab / 8, inner = spx < 4 ? spx : 4, groups = (spx + inner - 1) / inner;
    grid = 8 * groups * inner * p.nr;
  } else {
    grid = p.nslab * p.nr;
  }
  ffn_scatter_kernel<KS><<<grid, SC_THREADS, p.smem, st>>>(Hin, W, rstart, tok, s.N, s.d, s.T, p.R, p.nr,
                                                            p.nslab, out, Z);
  return hipGetLastError();
}

hipError_t launch_scatter(const spt_shape_t& s, const ScatterPlan& p, const uint16_t* Hin, const uint16_t* W,
                          const int32_t* rstart, const int32_t* tok, uint16_t* out, const uint16_t* Z,
                          hipStream_t st) {
  switch (s.Bs / 16) {
    case 2: return launch_scatter_t<2>(s, p, Hin, W, rstart, tok, out, Z, st);
    case 4: return launch_scatter_t<4>(s, p, Hin, W, rstart, tok, out, Z, st);
    case 6: return launch_scatter_t<6>(s, p, Hin, W, rstart, tok, out, Z, st);
    case 8: return launch_scatter_t<8>(s, p, Hin, W, rstart, tok, out, Z, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace spt
