// Grouped bf16 MFMA GEMMs of the routed FFN.
//
// Algorithm 4 of the paper runs, per weight block, a gather, two dense GEMMs and a scatter.
// Here every stage is ONE launch over all blocks: a row tile knows its bucket from a small
// prefix table built on the device, the gather is fused into the operand loads, and block
// outputs are added per token in a fixed order (in LDS for narrow blocks; through per-pair
// partial rows and a combine for wide ones).
//
// This file: the schedule tables, the K = d GEMMs of narrow blocks (up-projection + activation,
// dH * act'), the weight-gradient GEMMs (K = bucket rows), the combine used by the wide-block
// path, and the host-side sequencing of all stages.  The K = Bs contraction of narrow blocks
// (down-projection, dX) with Alg. 4's write-back folded in lives in ffn_scatter.hip; blocks
// wider than 128 units in ffn_wide.hip.
#include <stdlib.h>
#include <type_traits>

#include "ffn_common.hpp"
#include "spt_host.hpp"
#include "profile.hpp"

namespace spt {

// ------------------------------------------------------------------------------------------
// Schedule tables, built on the device from `offsets` by one workgroup (thread b = bucket b).
//
// The chip has 8 XCDs with a private L2 each, and workgroups are handed to XCDs round-robin
// by workgroup id, so "which XCD runs which tile, and when" decides what is served from L2
// and what has to come over the fabric.  Two tables:
//   border[N]         buckets by size, largest first (dW GEMMs start the long ones first);
//   kd_list[8][cap], kd_count[8]   per XCD, the row tiles of the K = d GEMMs in the order
//                     the XCD should run them.  With N >= 16 the buckets are dealt to the
//                     XCDs by size rank (boustrophedon, so the loads balance), and an XCD's
//                     list is ordered by tile level first (the i-th tile of every bucket it
//                     owns, which all cover the same window of token ids), bucket second:
//                     tiles that run together then share both the activation rows (each
//                     token sits in k of the N buckets) and, level after level, the same few
//                     weight blocks.  With fewer buckets the bucket-major tile sequence is
//                     cut into 8 contiguous runs (weight reuse only).

__global__ __launch_bounds__(1024) void plan_kernel(const int32_t* __restrict__ offsets, int N,
                                                    int QT, int cap,
                                                    int32_t* __restrict__ border,
                                                    int32_t* __restrict__ kd_count,
                                                    KdTile* __restrict__ kd_list,
                                                    uint32_t* __restrict__ zero_row,
                                                    const int32_t* __restrict__ perm, int P, int k,
                                                    int32_t* __restrict__ tok, int R, int nr,
                                                    int32_t* __restrict__ starts, int dw_rows, int dw_cap,
                                                    DwPiece* __restrict__ dw_pieces,
                                                    int32_t* __restrict__ dw_xlist) {
  // Workgroups past the first fill tok[q] = token of sorted position q (one launch instead of
  // two) and, for narrow blocks (R > 0), the table starts[r][b] = first sorted position of bucket
  // b whose token is >= r R (r = 0 .. nr): position q is that first position for every range
  // after its predecessor's and up to its own, and the bucket's end for the ranges behind its
  // last row -- every entry is written exactly once, no search, no atomics.
  if (blockIdx.x > 0) {
    __shared__ int32_t off_sh[1025];
    if (R > 0) {
      for (int e = threadIdx.x; e <= N; e += 1024) off_sh[e] = offsets[e];
      __syncthreads();
    }
    const int q = (blockIdx.x - 1) * 1024 + threadIdx.x;
    if (q >= P) return;
    const int t = perm[q] / k;
    tok[q] = t;
    if (R <= 0) return;
    int lo = 0, hi = N;   // bucket of q: the largest b with offsets[b] <= q
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (off_sh[mid] <= q) lo = mid; else hi = mid;
    }
    const int b = lo;
    const int rq = t / R;
    const int rprev = (q > off_sh[b]) ? (perm[q - 1] / k) / R : -1;
    for (int r = rprev + 1; r <= rq; ++r) starts[(size_t)r * N + b] = q;
    if (q + 1 == off_sh[b + 1])
      for (int r = rq + 1; r <= nr; ++r) starts[(size_t)r * N + b] = q + 1;
    return;
  }
  __shared__ int32_t scan[1024];
  if (threadIdx.x < 64) zero_row[threadIdx.x] = 0u;  // 256 bytes of zeros for padded K rows
  __shared__ int32_t sm_m[1024];
  __shared__ int32_t sm_ntq_by_rank[1024];
  const int b = threadIdx.x;
  const int off = (b < N) ? offsets[b] : 0;
  const int m = (b < N) ? offsets[b + 1] - off : 0;
  if (R > 0 && b < N && m == 0)   // an empty bucket has no row to write its table column
    for (int r = 0; r <= nr; ++r) starts[(size_t)r * N + b] = off;

  auto inclusive_scan = [&](int v) {
    __syncthreads();
    scan[b] = v;
    __syncthreads();
    for (int s = 1; s < 1024; s <<= 1) {
      const int t = (b >= s) ? scan[b - s] : 0;
      __syncthreads();
      scan[b] += t;
      __syncthreads();
    }
    return scan[b];
  };

  sm_m[b] = m;
  __syncthreads();
  int rank = 0;
  if (b < N)
    for (int o = 0; o < N; ++o) rank += (sm_m[o] > m) || (sm_m[o] == m && o < b);
  const int ntq = (m + QT - 1) / QT;
  if (b < N) {
    border[rank] = b;
    sm_ntq_by_rank[rank] = ntq;
  }
  __syncthreads();

  // Weight-gradient work items (backward, narrow blocks): a bucket of m rows becomes
  // ceil(m / dw_rows) pieces of equal size (an empty bucket one empty piece: its gradient block
  // is written as zeros), listed largest bucket first.  A bucket's first piece goes straight
  // into its gradient block, the others into staging slots that are added afterwards in order.
  if (dw_pieces) {
    __shared__ int32_t sm_np_rank[1024];
    __shared__ int32_t sm_wstart[1024];
    const int np = (b < N) ? (m > dw_rows ? (m + dw_rows - 1) / dw_rows : 1) : 0;
    const int x_end = inclusive_scan(np > 1 ? np - 1 : 0);     // staging slots, in bucket order
    const int l_end = inclusive_scan(np > 1 ? 1 : 0);          // buckets with staged pieces
    if (b < N && np > 1) {
      dw_xlist[1 + 3 * (l_end - 1)] = b;
      dw_xlist[2 + 3 * (l_end - 1)] = x_end - (np - 1);
      dw_xlist[3 + 3 * (l_end - 1)] = x_end;
    }
    if (b == N - 1) dw_xlist[0] = l_end;
    sm_np_rank[b] = 0;
    __syncthreads();
    if (b < N) sm_np_rank[rank] = np;
    __syncthreads();
    const int mine = sm_np_rank[b];
    const int w_end = inclusive_scan(mine);                    // work order: by rank
    sm_wstart[b] = w_end - mine;
    __shared__ int32_t total_pieces;
    if (b == 1023) total_pieces = w_end;
    __syncthreads();
    if (b < N) {
      const int at = sm_wstart[rank], base = m / np, rem = m % np;
      for (int pc = 0; pc < np; ++pc) {
        const int lo = off + pc * base + (pc < rem ? pc : rem);
        dw_pieces[at + pc] = DwPiece{lo, lo + base + (pc < rem ? 1 : 0), pc == 0 ? b : N + x_end - (np - 1) + pc - 1, 0};
      }
    }
    for (int e = total_pieces + b; e < dw_cap; e += 1024) dw_pieces[e] = DwPiece{0, 0, -1, 0};
  }

  if (N >= 16) {
    // rank r goes to group r%16 (<8) or 15 - r%16: position pg = r/8 inside the group; the
    // member at position p of group g has rank 8p + (p even ? g : 7 - g); sizes fall with p.
    const int pg = rank >> 3;
    const int g = (pg & 1) ? 7 - (rank & 7) : (rank & 7);
    auto member_ntq = [&](int grp, int p) {
      const int r = 8 * p + ((p & 1) ? 7 - grp : grp);
      return (r < N) ? sm_ntq_by_rank[r] : 0;
    };
    if (b < N) {
      int before = 0;             // tiles of lower levels in this group
      int alive = (N + 7) / 8;    // members that still have a tile at this level: a prefix
      for (int lvl = 0; lvl < ntq; ++lvl) {
        while (alive > 0 && member_ntq(g, alive - 1) <= lvl) --alive;
        kd_list[(size_t)g * cap + before + pg] = KdTile{b, off + lvl * QT};
        before += alive;
      }
    }
    if (b < 8) {
      int total = 0;
      for (int p = 0; 8 * p < N; ++p) total += member_ntq(b, p);
      kd_count[b] = total;
    }
  } else {
    const int inc = inclusive_scan(ntq);
    __shared__ int32_t total_sh;
    if (b == N - 1) total_sh = inc;
    __syncthreads();
    const int total = total_sh;
    const int per = (total + 7) / 8 > 0 ? (total + 7) / 8 : 1;
    if (b < N)
      for (int lvl = 0; lvl < ntq; ++lvl) {
        const int t = inc - ntq + lvl;
        kd_list[(size_t)(t / per) * cap + (t % per)] = KdTile{b, off + lvl * QT};
      }
    if (b < 8) {
      const int left = total - b * per;
      kd_count[b] = left < 0 ? 0 : (left < per ? left : per);
    }
  }
}

// ------------------------------------------------------------------------------------------
// K = d GEMM of one 256-row tile of one bucket for Bs <= 128, activation in the epilogue.
//   MODE 0 (forward, Alg. 4 line 4):  Hsave = Xg W1_b^T,  Hact = act(Hsave)
//   MODE 1 (backward):  dHpre = (dYg W2_b^T) * act'(Hsave),  Hact = act(Hsave)
// Hsave is row-major [P, Bs] (it crosses the ABI); Hact and dHpre are in fragment order (hfrag_off).
// C[u][q] is computed with hidden units as MFMA rows, so a lane holds, for ITS bucket row q,
// hidden units 8g + 4h + e of every 32-unit tile.  Four wavefronts own 64 bucket rows each
// (all hidden units) and share the LDS DMA: gathered rows + weight block through a 3-stage
// ring (global_load_lds_dwordx4, the gather folded into the DMA addresses).  The kernel is
// bound by bytes entering the CU; two workgroups per CU.  The K = Bs contraction that follows
// (down-projection, dX) is the token-range-stationary kernel of ffn_scatter.hip.
constexpr int KD_KT = 32;  // K values per stage
constexpr int FU_ROWS = 256;
constexpr int FU_STAGE1_SLOTS = (TILE + FU_ROWS) * 4;     // one stage: 24 KiB
constexpr int FU_SMEM_BYTES = 3 * FU_STAGE1_SLOTS * 16;   // 72 KiB

template <int MODE, int ACT, int KS>
__global__ __launch_bounds__(256, 2) void ffn_up_kernel(
    const uint16_t* __restrict__ Wa, const uint16_t* __restrict__ Act,
    const int32_t* __restrict__ offsets, const int32_t* __restrict__ kd_count,
    const KdTile* __restrict__ kd_list, int cap, const int32_t* __restrict__ tok, int Bs, int d,
    uint16_t* __restrict__ Hsave, uint16_t* __restrict__ Hact, uint16_t* __restrict__ dHpre,
    const uint16_t* __restrict__ Xe, const uint16_t* __restrict__ We) {
  constexpr int MI = KS / 2;   // 32-unit tiles of the block
  extern __shared__ uint4 fu_smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const uint32_t lds0 = (uint32_t)(uintptr_t)fu_smem;
  // Low-rank adapters (section 2.2) enter as two more K-stages: 64 extra K-values per
  // gathered row (Xe[token][64]) and per hidden unit (We[unit][64]).
  const int nkd = d / KD_KT;
  const int nk = nkd + (Xe ? 2 : 0);
  const int xcd = blockIdx.x & 7, wg_per_xcd = gridDim.x >> 3;
  const int count = kd_count[xcd];
  const int i = lane & 31, h = lane >> 5;
  for (int slot_id = blockIdx.x >> 3; slot_id < count; slot_id += wg_per_xcd) {
    const KdTile tile = kd_list[(size_t)xcd * cap + slot_id];
    const int b = tile.bucket, q0 = tile.q0;
    const int qend = offsets[b + 1];
    __builtin_amdgcn_s_barrier();  // LDS of the previous tile is free

    // DMA: a stage is 128 weight rows + 256 gathered rows of 64 bytes (32 K-values);
    // an instruction moves 16 rows; this wavefront issues 2 + 4 of the 8 + 16 per stage.
    // Lane L of instruction j fills row 16 j + L / 4, physical chunk L % 4 = logical ^ swizzle.
    // (the swizzle term (row >> 2) & 3 is (lane >> 4) & 3 for every instruction: the rows an
    // instruction covers start at a multiple of 16)
    const int ch8 = ((lane & 3) ^ ((lane >> 4) & 3)) * 8;
    int urow[2], tq[4];  // hidden unit / token id of this lane's row in each instruction
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int row = (wave * 2 + j) * 16 + (lane >> 2);
      urow[j] = b * Bs + (row < Bs ? row : 0);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int row = (wave * 4 + j) * 16 + (lane >> 2);
      tq[j] = tok[(q0 + row < qend) ? q0 + row : q0];
    }
    // (row addresses are formed once per tile: a 64-bit multiply per copy in the K loop sits on
    // the path between the barrier and the fragment reads)
    const uint16_t* arow[2];
    const uint16_t* brow[4];
#pragma unroll
    for (int j = 0; j < 2; ++j) arow[j] = Wa + (size_t)urow[j] * d + ch8;
#pragma unroll
    for (int j = 0; j < 4; ++j) brow[j] = Act + (size_t)tq[j] * d + ch8;
    // copy `piece` (0, 1: weight rows; 2 .. 5: gathered rows) of K-stage kt into ring slot `stage`
    auto issue_piece = [&](int stage, int kt, int piece) {
      const uint32_t base = lds0 + (uint32_t)(stage * FU_STAGE1_SLOTS) * 16u;
      const bool ext = kt >= nkd;  // wave-uniform
      if (piece < 2) {
        const int j = piece;
        dma16(ext ? We + (size_t)urow[j] * (2 * KD_KT) + ch8 + (kt - nkd) * KD_KT : arow[j] + kt * KD_KT,
              __builtin_amdgcn_readfirstlane(base + (uint32_t)((wave * 2 + j) * 64) * 16u));
      } else {
        const int j = piece - 2;
        dma16(ext ? Xe + (size_t)tq[j] * (2 * KD_KT) + ch8 + (kt - nkd) * KD_KT : brow[j] + kt * KD_KT,
              __builtin_amdgcn_readfirstlane(base + (uint32_t)(TILE * 4 + (wave * 4 + j) * 64) * 16u));
      }
    };

    f32x16 acc[MI][2];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < 2; ++ni)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;
    // Ring schedule: "issue j" copies K-stage min(j, nk-1) into slot j % 3; past the last stage it
    // repeats it into a slot nobody reads any more, so the loop body has no branch and every
    // vmcnt wait is a constant.  Issues 0 and 1 go out up front, iteration kt sends issue kt+2
    // piece by piece behind its first MFMAs (the slot stage kt-1 left at the barrier).
    const int klast = nk - 1;
#pragma unroll
    for (int p6 = 0; p6 < 6; ++p6) issue_piece(0, 0, p6);
#pragma unroll
    for (int p6 = 0; p6 < 6; ++p6) issue_piece(1, klast < 1 ? klast : 1, p6);
    int stage = 0;
    for (int kt = 0; kt < nk; ++kt) {
      // own copies of stage kt have landed (stage kt+1's six may still be in flight) ...
      wait_vmcnt<6>();
      __builtin_amdgcn_s_barrier();  // ... and everyone's; all are done reading stage kt-1
      const int fill = stage >= 1 ? stage - 1 : 2;
      const int kfill = kt + 2 < klast ? kt + 2 : klast;
      const uint4* As = fu_smem + stage * FU_STAGE1_SLOTS;
      const uint4* Bt = As + TILE * 4;
      // all fragment reads of the stage go out first, so the MFMAs of the first K-step run
      // while the second K-step's fragments are still arriving (the compiler left to itself
      // sinks each read next to its use and exposes the LDS latency every few MFMAs)
      bf16x8 a[KD_KT / 16][MI], bb[KD_KT / 16][2];
#pragma unroll
      for (int s = 0; s < KD_KT / 16; ++s) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) a[s][mi] = as_bf16x8(As[kd_slot(mi * 32 + i, 2 * s + h)]);
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) bb[s][ni] = as_bf16x8(Bt[kd_slot(wave * 64 + ni * 32 + i, 2 * s + h)]);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int s = 0; s < KD_KT / 16; ++s)
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
          for (int ni = 0; ni < 2; ++ni) {
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[s][mi], bb[s][ni], acc[mi][ni], 0, 0, 0);
            const int m = (s * MI + mi) * 2 + ni;
            if (m < 6) {
              issue_piece(fill, kfill, m);
              __builtin_amdgcn_sched_barrier(0);
            }
          }
#pragma unroll
      for (int m = (KD_KT / 16) * MI * 2; m < 6; ++m) issue_piece(fill, kfill, m);  // 32-unit blocks: 4 MFMAs only
      __builtin_amdgcn_sched_barrier(0);
      stage = (stage == 2) ? 0 : stage + 1;
    }
    wait_vmcnt<0>();  // the trailing copies (repeats of the last stage) are done too
    // epilogue: lane (i, h) holds, for row q, units 32 mi + 8 g + 4 h + e  (v = 4 g + e)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) {
      const int q = q0 + wave * 64 + ni * 32 + i;
      const bool live = q < qend;
      const size_t orow = (size_t)(live ? q : q0) * Bs;
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const size_t off = orow + mi * 32 + 8 * g + 4 * h;                        // Hsave: row-major
          const size_t foff = hfrag_off(live ? q : q0, mi * 32 + 8 * g + 4 * h, Bs);  // Hact, dHpre
          const float c0 = acc[mi][ni][4 * g], c1 = acc[mi][ni][4 * g + 1];
          const float c2 = acc[mi][ni][4 * g + 2], c3 = acc[mi][ni][4 * g + 3];
          if (MODE == 0) {
            if (live) {
              if (Hsave)
                *reinterpret_cast<uint2*>(Hsave + off) = make_uint2(pack_bf16x2(c0, c1), pack_bf16x2(c2, c3));
              *reinterpret_cast<uint2*>(Hact + foff) =
                  make_uint2(pack_bf16x2(act_fn<ACT>(c0), act_fn<ACT>(c1)),
                             pack_bf16x2(act_fn<ACT>(c2), act_fn<ACT>(c3)));
            }
          } else {
            const uint2 hp = *reinterpret_cast<const uint2*>(Hsave + off);
            const float z0 = lo_bf16(hp.x), z1 = hi_bf16(hp.x), z2 = lo_bf16(hp.y), z3 = hi_bf16(hp.y);
            if (live) {
              *reinterpret_cast<uint2*>(dHpre + foff) =
                  make_uint2(pack_bf16x2(c0 * act_grad<ACT>(z0), c1 * act_grad<ACT>(z1)),
                             pack_bf16x2(c2 * act_grad<ACT>(z2), c3 * act_grad<ACT>(z3)));
              *reinterpret_cast<uint2*>(Hact + foff) =
                  make_uint2(pack_bf16x2(act_fn<ACT>(z0), act_fn<ACT>(z1)),
                             pack_bf16x2(act_fn<ACT>(z2), act_fn<ACT>(z3)));
            }
          }
        }
        // keep the scheduler from interleaving the 16-value groups: their erf evaluations
        // would otherwise all be in flight at once and spill
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// K = bucket rows GEMMs for Bs <= 128: dW1 (Act = X, Hin = dHpre) and dW2 (Act = dY, Hin = act(H)).
//   dW[b][u][c] = sum_{q in bucket b} Hin[q][u] * Act[tok[q]][c]    MFMA rows c, columns u
// K runs over the bucket's rows in sorted order, so the sum order is fixed (no split-K, no
// atomics).  A workgroup owns CT output columns x UT hidden units of one block (CT = 256 here; 512
// further down).  UT = 128: wavefront (wm, wn) owns 128 columns x 64 units (4 x 2 MFMA tiles);
// UT = 64, for blocks of at most 64 units (a 128-unit tile would be half padding): wavefront wm
// owns 64 columns x 64 units (2 x 2 tiles).  Two workgroups share a CU.
// Both operands are token-major in memory, i.e. K is the strided dimension for both.  They
// are copied as they are into a 6-slot LDS ring (16 tokens per stage: 16 x 512 B of gathered
// activation columns + 16 x 256 B of Hin) by global_load_lds_dwordx4, and ds_read_b64_tr_b16
// builds the K-contiguous MFMA fragments out of the token-major tiles; the column side goes
// through the rho32 row permutation, so a lane ends up with 16 consecutive columns of one
// hidden unit (64-byte runs of fp32; the epilogue regroups them into whole lines through LDS).
// Ring schedule: "issue j" copies stage min(j, nk-1) into slot j % 6 (past the last stage it
// repeats it into a slot nobody reads: the loop body has no branch and every vmcnt wait is a
// constant).  Issues 0..4 go out up front, iteration kt sends issue kt+5 (LA = 5 below).  At the top of
// iteration kt the stages kt and kt+1 are visible and the fragments of stage kt are in
// registers; the iteration multiplies them (8 MFMAs per wavefront) with, behind each MFMA, one
// piece of the other work: first the 3 DMA instructions (the copies are what the kernel waits
// for, so the slot the barrier has just freed is refilled at once: sending them last cost 4 %) and
// the scalar loads of the token ids for the next iteration's DMA (wave-uniform addresses in the
// constant address space; they leave the vmcnt bookkeeping alone), then the 6 fragment reads of
// stage kt+1.
// Rows past the bucket's end read a zero line for Hin (so they add nothing) and any valid row
// for the activations.
//
// CT = 512: eight wavefronts share one workgroup's hidden-unit tiles for two 256-column halves (one
// workgroup per CU; the same wavefronts per CU, tiles per wavefront and registers as two workgroups
// of four).  The hidden-unit side is then copied once for 512 columns instead of once per 256: a
// sixth fewer bytes into the CU, which is what the kernel waits for.  Wavefronts 4-7 copy the second
// half's columns of the same token rows and no hidden-unit rows.
constexpr int DW_KT = 16;                          // tokens per stage
constexpr int DW_HALF_BYTES = DW_KT * 256 * 2;     // 8 KiB: 16 token rows x 256 columns
constexpr int DW_SLOTS = 6;   // 72 KiB per workgroup with 256 x 128 tiles, 120 with 512 x 128 (a 7th slot gained nothing)

template <bool FRAG, int UT, int CT>  // FRAG: Hin in fragment order (hfrag_off) instead of row-major [rows, Bs]
__global__ __launch_bounds__(CT, CT == 512 ? 1 : 2) void kq_gemm_kernel(
    const uint16_t* __restrict__ Act, const uint16_t* __restrict__ Hin,
    const int32_t* __restrict__ offsets, const int32_t* __restrict__ tok,
    const int32_t* __restrict__ border, const uint16_t* __restrict__ zero_row, int N, int Bs,
    int d, float* __restrict__ dW, const DwPiece* __restrict__ pieces, int nblocks,
    float* __restrict__ stage) {
  constexpr int MI = UT == 128 ? 4 : 2;               // 32-column tiles per wavefront
  constexpr int DW_CT = CT;
  constexpr int DW_A_BYTES = (CT / 256) * DW_HALF_BYTES;   // 8 or 16 KiB
  constexpr int DW_B_BYTES = DW_KT * UT * 2;          // 4 or 2 KiB
  constexpr int DW_STAGE_BYTES = DW_A_BYTES + DW_B_BYTES;
  constexpr int CPW = UT == 128 ? 128 : 64;           // columns per wavefront
  constexpr int LA = DW_SLOTS - 1;                    // stages a copy is issued ahead of its use
  extern __shared__ uint4 dw_smem[];
  // Work item = (column tile, bucket).  An XCD (workgroup id mod 8) keeps to its own column
  // tiles and walks the buckets, largest first: the workgroups that run together on an XCD
  // then gather the same narrow column slab of the activations -- it fits that XCD's L2 and
  // every token row in it is wanted by k of the N buckets.
  const int nct = (d + DW_CT - 1) / DW_CT;
  const int xcd = blockIdx.x & 7, jj = blockIdx.x >> 3;
  int ct, br;
  if (nct % 8 == 0) {
    const int per = nct / 8;
    ct = xcd + 8 * (jj % per);
    br = jj / per;
  } else if (8 % nct == 0) {
    const int r = 8 / nct;
    ct = xcd % nct;
    br = xcd / nct + r * jj;
  } else {
    ct = blockIdx.x % nct;
    br = blockIdx.x / nct;
  }
  if (br >= N) return;   // N: work items (buckets, or entries of the piece table)
  int qb, qe;
  float* dst;
  if (pieces) {
    const DwPiece pc = pieces[br];
    if (pc.dst < 0) return;
    qb = pc.lo; qe = pc.hi;
    dst = pc.dst < nblocks ? dW + (size_t)pc.dst * Bs * d : stage + (size_t)(pc.dst - nblocks) * Bs * d;
  } else {
    const int b = border[br];
    qb = offsets[b]; qe = offsets[b + 1];
    dst = dW + (size_t)b * Bs * d;
  }
  const int c0 = ct * DW_CT, u0 = blockIdx.y * UT;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = UT == 128 ? wave >> 1 : wave, wn = UT == 128 ? wave & 1 : 0;
  const int wq = wave & 3, chalf = wave >> 2;          // copy role: quarter of the token rows, column half
  const int fhalf = (wm * CPW) >> 8, fwm = wm & (256 / CPW - 1);  // fragment role: column half, place in it
  const bool copies_b = wave < 4;
  const int i = lane & 31, h = lane >> 5;
  const uint32_t lds0 = (uint32_t)(uintptr_t)dw_smem;
  const int nk = (qe - qb + DW_KT - 1) / DW_KT;
  const int klast = nk - 1;

  // DMA lane roles.  Activations: instruction j (2 per wavefront) moves token rows
  // 4 wave + 2j, + 1 of the stage, 512 B each: lane L -> row + L/32, physical chunk L%32 =
  // logical ^ ((row&3)<<2).  Hin, UT = 128: one instruction per wavefront moves rows 4 wave .. + 3,
  // 256 B each: lane L -> row 4 wave + L/16, physical chunk L%16 = logical ^ ((row&3)<<2).  UT = 64:
  // an instruction moves 8 rows of 128 B (lane L -> row + L/8, physical chunk L%8 = logical ^
  // (((row>>1)&1)<<2)); wavefronts 2 and 3 repeat the copies of 0 and 1 -- same bytes to the same
  // place -- so that every wavefront has the same number of copies in flight.
  const int lane_half = lane >> 5;
  int a_coloff[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int row = 4 * wq + 2 * j + lane_half;
    const int col = c0 + 256 * chalf + (((lane & 31) ^ ((row & 3) << 2)) << 3);
    a_coloff[j] = (col < d) ? col : c0;  // ragged last column tile: harmless duplicate, never stored
  }
  const int b_row = UT == 128 ? 4 * wq + (lane >> 4) : 8 * (wave & 1) + (lane >> 3);
  int b_coloff = UT == 128 ? u0 + (((lane & 15) ^ ((b_row & 3) << 2)) << 3)
                           : u0 + (((lane & 7) ^ (((b_row >> 1) & 1) << 2)) << 3);
  if (b_coloff >= Bs) b_coloff = u0;
  typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;
  const const_i32_ptr tok_c = (const_i32_ptr)(uintptr_t)tok;
  auto load_ids = [&](int kt, int (&ids)[4]) {  // token ids of this wavefront's 4 rows of stage kt
    const int r0 = qb + kt * DW_KT + 4 * wq;
#pragma unroll
    for (int e = 0; e < 4; ++e) ids[e] = tok_c[min(r0 + e, qe - 1)];
  };
  auto issue_a = [&](int j, int slot, const int (&ids)[4]) {
    // (arithmetic select: a select between two array elements would become an indexed load
    // from a private-memory copy of the array)
    const int t = ids[2 * j] + lane_half * (ids[2 * j + 1] - ids[2 * j]);
    dma16(Act + (size_t)t * d + a_coloff[j],
          __builtin_amdgcn_readfirstlane(
              lds0 + (uint32_t)(slot * DW_STAGE_BYTES + chalf * DW_HALF_BYTES + (wq * 2 + j) * 1024)));
  };
  auto issue_b = [&](int slot, int kt) {
    if (CT == 512 && !copies_b) return;  // (wave-uniform)
    const int q = qb + kt * DW_KT + b_row;
    const uint16_t* src = (q < qe) ? Hin + hval_off<FRAG>(q, b_coloff, Bs) : zero_row + ((lane & 15) << 3);
    dma16(src, __builtin_amdgcn_readfirstlane(
                   lds0 + (uint32_t)(slot * DW_STAGE_BYTES + DW_A_BYTES + (UT == 128 ? wq : wave & 1) * 1024)));
  };

  // Transposing fragment reads, lane (group g = lane/16, s = lane%16): token row
  // 8 (g>>1) + 4 r + (s>>2) of the stage; column group: the rho32-permuted one on the column
  // side (4 * colgrp), natural order 16 (g&1) + 4 (s&3) on the hidden-unit side.
  const int g = lane >> 4, sl = lane & 15;
  const int sw = ((sl >> 2) & 3) << 2;  // ((krow & 3) << 2): krow & 3 = (s >> 2) & 3
  const int ag = sl & 3;
  const int acol = 4 * (4 * (ag & 1) + 2 * (g & 1) + (ag >> 1));
  const int bcol = 16 * (g & 1) + 4 * (sl & 3);
  const int krow0 = 8 * (g >> 1) + (sl >> 2);
  const int swb = UT == 128 ? sw : ((krow0 >> 1) & 1) << 2;
  uint32_t a_off[MI], b_off[2];  // byte offsets of the r = 0 read inside a stage
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
    a_off[mi] = (uint32_t)(fhalf * DW_HALF_BYTES + krow0 * 512 + ((((fwm * MI + mi) * 4 + (acol >> 3)) ^ sw) * 16) +
                           (acol & 4) * 2);
#pragma unroll
  for (int ni = 0; ni < 2; ++ni)
    b_off[ni] = (uint32_t)(DW_A_BYTES + krow0 * (2 * UT) + ((((wn * 2 + ni) * 4 + (bcol >> 3)) ^ swb) * 16) + (bcol & 4) * 2);
  const char* ring = reinterpret_cast<const char*>(dw_smem);
  auto load_frag = [&](const char* st, int f) -> bf16x8 {  // f < MI: column tile f; else unit tile f - MI
    if (f < MI) return tr_read_frag(st + a_off[f], st + a_off[f] + 4 * 512);
    return tr_read_frag(st + b_off[f - MI], st + b_off[f - MI] + 4 * (2 * UT));
  };

  f32x16 acc[MI][2];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;

  bf16x8 fa[2][MI], fb[2][2];
  int ids[4] = {0, 0, 0, 0};
  if (nk > 0) {
#pragma unroll
    for (int st = 0; st < LA; ++st) {
      const int ks = st < klast ? st : klast;
      load_ids(ks, ids);
      issue_a(0, st, ids);
      issue_a(1, st, ids);
      issue_b(st, ks);
    }
    load_ids(LA < klast ? LA : klast, ids);
    // issues 0 and 1 have landed (the LA - 2 later ones may be out: 3 instructions each, 2 without hidden rows)
    if (CT == 512 && !copies_b) wait_vmcnt<2 * (LA - 2)>(); else wait_vmcnt<3 * (LA - 2)>();
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int f = 0; f < MI; ++f) fa[0][f] = load_frag(ring, f);
#pragma unroll
    for (int f = 0; f < 2; ++f) fb[0][f] = load_frag(ring, f + MI);
  }
  // One iteration; cur says which fragment buffer holds stage kt (a compile-time constant, so
  // the buffers stay in registers: the loop below is unrolled by two).
  auto iteration = [&](int kt, int slot, auto cur_tag) {
    constexpr int cur = decltype(cur_tag)::value;
    const int next_slot = (slot + 1 == DW_SLOTS) ? 0 : slot + 1;
    const int fill = (slot == 0) ? DW_SLOTS - 1 : slot - 1;  // slot of stage kt-1 = that of stage kt+LA
    // after the last stage the look-ahead reads the current one again: harmless
    const char* st1 = ring + ((kt + 1 < nk) ? next_slot : slot) * DW_STAGE_BYTES;
    const int kfill = kt + LA < klast ? kt + LA : klast;
    int ids_next[4] = {0, 0, 0, 0};
#pragma unroll
    for (int m = 0; m < 2 * MI; ++m) {
      const int mi = m >> 1, ni = m & 1;
      acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur][mi], fb[cur][ni], acc[mi][ni], 0, 0, 0);
      if (m == 0) { issue_a(0, fill, ids); issue_a(1, fill, ids); }
      else if (m == 1) { issue_b(fill, kfill); load_ids(kt + LA + 1 < klast ? kt + LA + 1 : klast, ids_next); }
      else if (m < MI + 2) fa[cur ^ 1][m - 2] = load_frag(st1, m - 2);
      else fb[cur ^ 1][m - MI - 2] = load_frag(st1, m - 2);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (2 * MI < MI + 4) {  // 64-unit tiles: 4 MFMAs only, the hidden-unit fragments follow them
      fb[cur ^ 1][0] = load_frag(st1, MI);
      fb[cur ^ 1][1] = load_frag(st1, MI + 1);
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) ids[e] = ids_next[e];
    // own copies of stage kt+2 have landed: only issues kt+3 .. kt+LA (3 instructions each) may
    // be outstanding; the barrier makes everyone's visible and ends all reads of stage kt
    if (CT == 512 && !copies_b) wait_vmcnt<2 * (LA - 2)>(); else wait_vmcnt<3 * (LA - 2)>();
    __builtin_amdgcn_s_barrier();
  };
  int slot = 0;
  for (int kt = 0; kt < nk; kt += 2) {
    iteration(kt, slot, std::integral_constant<int, 0>{});
    slot = (slot + 1 == DW_SLOTS) ? 0 : slot + 1;
    if (kt + 1 < nk) {
      iteration(kt + 1, slot, std::integral_constant<int, 1>{});
      slot = (slot + 1 == DW_SLOTS) ? 0 : slot + 1;
    }
  }
  wait_vmcnt<0>();  // the trailing copies (repeats of the last stage) are done too
  __builtin_amdgcn_s_barrier();  // ... everyone's: the ring is free

  // Lane (i, h) holds, for hidden unit u0 + 64 wn + 32 ni + i, the columns
  // c0 + 32 MI wm + 32 mi + 16 h + (0..15): stored as they are, an instruction would touch 64
  // lines with 16 bytes each.  Each 32 x 32 tile goes through a wavefront-private LDS buffer
  // (rows of 144 bytes) instead, and comes back with 8 lanes along a row, so a store instruction
  // writes 8 whole 128-byte lines.  (Same wavefront on both sides: LDS executes its accesses in order.)
  float* tbuf = reinterpret_cast<float*>(dw_smem) + wave * (32 * 36);
  const int cc = lane & 7, r0 = lane >> 3;
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) {
      const f32x16& v = acc[mi][ni];
#pragma unroll
      for (int e = 0; e < 4; ++e)
        *reinterpret_cast<f32x4*>(tbuf + i * 36 + 16 * h + 4 * e) = f32x4{v[4 * e], v[4 * e + 1], v[4 * e + 2], v[4 * e + 3]};
      wave_lds_fence();
      const int c = c0 + wm * CPW + mi * 32 + 4 * cc;
      f32x4 o[4];  // (all four reads go out before the first store waits for its data)
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = *reinterpret_cast<const f32x4*>(tbuf + (r0 + 8 * e) * 36 + 4 * cc);
      wave_lds_fence();
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int u = u0 + wn * 64 + ni * 32 + r0 + 8 * e;
        if (u < Bs && c < d) *reinterpret_cast<f32x4*>(dst + (size_t)u * d + c) = o[e];
      }
    }
}

// dW[b] += stage[first] + ... + stage[end - 1] (in that order) for every bucket b that was cut
// into more than one piece; xlist = (count, then (bucket, first slot, end slot) triples).
__global__ __launch_bounds__(256) void dw_reduce_kernel(float* __restrict__ dW, const float* __restrict__ stage,
                                                        const int32_t* __restrict__ xlist, int Bs, int d) {
  const int count = xlist[0];
  const size_t e4 = (size_t)Bs * d / 4;   // 16-byte groups per block
  for (size_t it = (size_t)blockIdx.x * 256 + threadIdx.x; it < (size_t)count * e4;
       it += (size_t)gridDim.x * 256) {
    const int l = (int)(it / e4);
    const size_t e = it % e4;
    const int b = xlist[1 + 3 * l], first = xlist[2 + 3 * l], end = xlist[3 + 3 * l];
    f32x4* acc = reinterpret_cast<f32x4*>(dW + (size_t)b * Bs * d) + e;
    f32x4 v = *acc;
    for (int x = first; x < end; ++x) v += reinterpret_cast<const f32x4*>(stage + (size_t)x * Bs * d)[e];
    *acc = v;
  }
}

// ------------------------------------------------------------------------------------------
// Combine: out[t][:] = sum_{j<k} part[inv[t*k+j]][:], j ascending, fp32, one rounding to bf16.
// This is Alg. 4's write-back with block outputs added (k > 1 blocks per token).
// `part` holds dc columns per row: column c of row r sits at r*row_stride + (c/128)*chunk_stride
// + c%128 (row-major: row_stride = dc, chunk_stride = 128; chunk-major, the layout the
// row-walking GEMM writes as whole contiguous 32 KiB blocks: row_stride = 128, chunk_stride =
// P*128).  `out` points at the first of those columns inside the [T, out_ld] result.
__global__ __launch_bounds__(256) void combine_kernel(const uint16_t* __restrict__ part,
                                                      const int32_t* __restrict__ inv, int T, int dc,
                                                      size_t row_stride, size_t chunk_stride,
                                                      int out_ld, int k,
                                                      uint16_t* __restrict__ out,
                                                      const uint16_t* __restrict__ Z) {
  const int cpr = dc >> 3;  // 16-byte groups per row
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= (int64_t)T * cpr) return;
  const int t = (int)(gid / cpr), cg = (int)(gid % cpr);
  float a[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) a[e] = 0.f;
  const int32_t* iv = inv + (size_t)t * k;
  part += (size_t)(cg >> 4) * chunk_stride + (cg & 15) * 8;
  int j = 0;
  for (; j + 8 <= k; j += 8) {
    u32x4 v[8];
#pragma unroll
    for (int jj = 0; jj < 8; ++jj)
      v[jj] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(part + (size_t)iv[j + jj] * row_stride));
#pragma unroll
    for (int jj = 0; jj < 8; ++jj) {
      a[0] += lo_bf16(v[jj].x); a[1] += hi_bf16(v[jj].x);
      a[2] += lo_bf16(v[jj].y); a[3] += hi_bf16(v[jj].y);
      a[4] += lo_bf16(v[jj].z); a[5] += hi_bf16(v[jj].z);
      a[6] += lo_bf16(v[jj].w); a[7] += hi_bf16(v[jj].w);
    }
  }
  for (; j < k; ++j) {
    const uint4 v = *reinterpret_cast<const uint4*>(part + (size_t)iv[j] * row_stride);
    a[0] += lo_bf16(v.x); a[1] += hi_bf16(v.x);
    a[2] += lo_bf16(v.y); a[3] += hi_bf16(v.y);
    a[4] += lo_bf16(v.z); a[5] += hi_bf16(v.z);
    a[6] += lo_bf16(v.w); a[7] += hi_bf16(v.w);
  }
  if (Z) {  // one more row per token: the low-rank term of the outer projection (section 2.2)
    const uint4 v = *reinterpret_cast<const uint4*>(Z + (size_t)t * out_ld + cg * 8);
    a[0] += lo_bf16(v.x); a[1] += hi_bf16(v.x);
    a[2] += lo_bf16(v.y); a[3] += hi_bf16(v.y);
    a[4] += lo_bf16(v.z); a[5] += hi_bf16(v.z);
    a[6] += lo_bf16(v.w); a[7] += hi_bf16(v.w);
  }
  *reinterpret_cast<uint4*>(out + (size_t)t * out_ld + cg * 8) =
      make_uint4(pack_bf16x2(a[0], a[1]), pack_bf16x2(a[2], a[3]), pack_bf16x2(a[4], a[5]),
                 pack_bf16x2(a[6], a[7]));
}

// ------------------------------------------------------------------------------------------
// host side
static int max_row_tiles(const spt_shape_t& s, int rows) {
  const int64_t P = (int64_t)s.T * s.k;
  return (int)((P + rows - 1) / rows) + s.N;
}

static bool use_narrow(const spt_shape_t& s) { return s.Bs <= TILE; }

static size_t carve_schedule(const spt_shape_t& s, char* p, size_t o0, Schedule& sc, bool weight_grads = false) {
  const size_t P = (size_t)s.T * s.k;
  size_t o = o0;
  sc.kd_cap = max_row_tiles(s, FU_ROWS);  // the narrow- and wide-block kernels both walk 256-row tiles
  sc.border = reinterpret_cast<int32_t*>(p + o);      o += align256((size_t)s.N * 4);
  sc.kd_count = reinterpret_cast<int32_t*>(p + o);    o += align256(8 * 4);
  sc.kd_list = p + o;                                 o += align256((size_t)8 * sc.kd_cap * sizeof(KdTile));
  sc.tok = reinterpret_cast<int32_t*>(p + o);         o += align256(P * 4);
  sc.zero_row = reinterpret_cast<uint16_t*>(p + o);   o += 256;
  sc.rstart = nullptr;
  if (use_narrow(s)) {
    sc.rstart = reinterpret_cast<int32_t*>(p + o);    o += plan_scatter(s).table_bytes;
  }
  sc.dw_pieces = nullptr; sc.dw_xlist = nullptr; sc.dw_cap = 0; sc.dw_rows = 0;
  if (use_narrow(s) && weight_grads) {
    // pieces of at most 1.5 x the mean bucket (never below 256 rows): balanced routing is left
    // alone, a bucket several times the mean no longer holds up the whole launch
    const int64_t mean15 = (3 * (int64_t)P / s.N + 1) / 2;
    sc.dw_rows = (int)((mean15 < 256 ? 256 : mean15) + 15) / 16 * 16;
    sc.dw_cap = s.N + (int)(P / sc.dw_rows);
    sc.dw_pieces = reinterpret_cast<DwPiece*>(p + o);  o += align256((size_t)sc.dw_cap * sizeof(DwPiece));
    sc.dw_xlist = reinterpret_cast<int32_t*>(p + o);   o += align256((size_t)(1 + 3 * s.N) * 4);
  }
  return o - o0;
}

static size_t hrows(size_t P) { return (P + 31) / 32 * 32; }  // rows of a tensor in fragment order

// Partial rows exist only on the wide-block path.
static size_t carve_part(const spt_shape_t& s, char* p, size_t o0, uint16_t*& part) {
  part = nullptr;
  if (use_narrow(s)) return 0;
  part = reinterpret_cast<uint16_t*>(p + o0);
  return align256((size_t)s.T * s.k * (size_t)s.d * 2);
}

FwdWorkspace plan_fwd(const spt_shape_t& s, void* ws) {
  const size_t P = (size_t)s.T * s.k;
  char* p = static_cast<char*>(ws);
  size_t o = 0;
  FwdWorkspace w;
  o += carve_schedule(s, p, o, w.sched);
  w.Hact = reinterpret_cast<uint16_t*>(p + o);       o += align256(hrows(P) * s.Bs * 2);
  o += carve_part(s, p, o, w.part);
  w.bytes = o;
  return w;
}

BwdWorkspace plan_bwd(const spt_shape_t& s, void* ws, bool weight_grads) {
  const size_t P = (size_t)s.T * s.k;
  char* p = static_cast<char*>(ws);
  size_t o = 0;
  BwdWorkspace w;
  o += carve_schedule(s, p, o, w.sched, weight_grads);
  w.Hact = reinterpret_cast<uint16_t*>(p + o);       o += align256(hrows(P) * s.Bs * 2);
  w.dHpre = reinterpret_cast<uint16_t*>(p + o);      o += align256(hrows(P) * s.Bs * 2);
  o += carve_part(s, p, o, w.part);
  w.dw_stage = nullptr;
  if (w.sched.dw_cap > 0) {
    w.dw_stage = reinterpret_cast<float*>(p + o);
    o += align256((size_t)(w.sched.dw_cap - s.N) * s.Bs * s.d * 4);
  }
  w.bytes = o;
  return w;
}

size_t schedule_bytes(const spt_shape_t& s) {
  Schedule sc;
  return carve_schedule(s, nullptr, 0, sc, true);
}

Schedule plan_schedule(const spt_shape_t& s, void* buf) {
  Schedule sc;
  carve_schedule(s, static_cast<char*>(buf), 0, sc, true);
  return sc;
}

#define SPT_LAUNCH_CHECK()                 \
  do {                                     \
    hipError_t e_ = hipGetLastError();     \
    if (e_ != hipSuccess) return e_;       \
  } while (0)

static hipError_t run_plan(const spt_shape_t& s, const int32_t* offsets, const int32_t* perm,
                           const Schedule& sc, hipStream_t st) {
  const int P = s.T * s.k;
  const ScatterPlan sp = sc.rstart ? plan_scatter(s) : ScatterPlan{};
  {
    ScopedKernelTimer tm(kSlotPlan, st);
    plan_kernel<<<1 + (P + 1023) / 1024, 1024, 0, st>>>(offsets, s.N, FU_ROWS, sc.kd_cap, sc.border, sc.kd_count,
                                                        static_cast<KdTile*>(sc.kd_list),
                                                        reinterpret_cast<uint32_t*>(sc.zero_row), perm, P, s.k,
                                                        sc.tok, sc.rstart ? sp.R : 0, sp.nr,
                                                        sc.rstart ? scatter_starts(sp, sc.rstart) : nullptr,
                                                        sc.dw_rows, sc.dw_cap, sc.dw_pieces, sc.dw_xlist);
  }
  SPT_LAUNCH_CHECK();
  if (sc.rstart) {
    ScopedKernelTimer tm(kSlotPlan, st);
    return run_scatter_ranges(s, sp, sc.rstart, st);
  }
  return hipSuccess;
}

hipError_t run_schedule(const spt_shape_t& s, const int32_t* offsets, const int32_t* perm, const Schedule& sc,
                        hipStream_t st) {
  return run_plan(s, offsets, perm, sc, st);
}

static hipError_t run_combine(const spt_shape_t& s, const uint16_t* part, const int32_t* inv,
                              void* out, int c_begin, int dc, size_t row_stride,
                              size_t chunk_stride, int slot, hipStream_t st,
                              const uint16_t* Z = nullptr) {
  const int64_t items = (int64_t)s.T * (dc / 8);
  ScopedKernelTimer tm(slot, st);
  combine_kernel<<<(unsigned)((items + 255) / 256), 256, 0, st>>>(
      part, inv, s.T, dc, row_stride, chunk_stride, s.d, s.k, static_cast<uint16_t*>(out) + c_begin,
      Z ? Z + c_begin : nullptr);
  SPT_LAUNCH_CHECK();
  return hipSuccess;
}

template <int MODE, int ACT, int KS>
static hipError_t launch_up_t(const spt_shape_t& s, const uint16_t* Wa, const uint16_t* Act,
                              const int32_t* offsets, const Schedule& sc, uint16_t* Hsave, uint16_t* Hact,
                              uint16_t* dHpre, hipStream_t st, const uint16_t* Xe, const uint16_t* We) {
  static bool attr_set = false;
  if (!attr_set) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(ffn_up_kernel<MODE, ACT, KS>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, FU_SMEM_BYTES);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int wg_per_xcd = sc.kd_cap < 64 ? sc.kd_cap : 64;  // two workgroups per CU
  ffn_up_kernel<MODE, ACT, KS><<<dim3(8 * wg_per_xcd), 256, FU_SMEM_BYTES, st>>>(
      Wa, Act, offsets, sc.kd_count, static_cast<const KdTile*>(sc.kd_list), sc.kd_cap, sc.tok, s.Bs, s.d,
      Hsave, Hact, dHpre, Xe, We);
  return hipGetLastError();
}

// K = d GEMM of the narrow-block path.  MODE 0: Hsave (may be null), Hact from Act = X, Wa = W1;
// MODE 1: dHpre, Hact from Act = dY, Wa = W2 and the forward's Hsave.
template <int MODE>
static hipError_t launch_up(const spt_shape_t& s, const uint16_t* Wa, const uint16_t* Act,
                            const int32_t* offsets, const Schedule& sc, uint16_t* Hsave, uint16_t* Hact,
                            uint16_t* dHpre, hipStream_t st, const uint16_t* Xe = nullptr,
                            const uint16_t* We = nullptr) {
#define SPT_UP(ACT, KS) return launch_up_t<MODE, ACT, KS>(s, Wa, Act, offsets, sc, Hsave, Hact, dHpre, st, Xe, We)
#define SPT_UP_KS(ACT)                    \
  switch (s.Bs / 16) {                    \
    case 2: SPT_UP(ACT, 2);               \
    case 4: SPT_UP(ACT, 4);               \
    case 6: SPT_UP(ACT, 6);               \
    default: SPT_UP(ACT, 8);              \
  }
  if (s.act == SPT_ACT_GELU) { SPT_UP_KS(0) } else { SPT_UP_KS(1) }
#undef SPT_UP_KS
#undef SPT_UP
}

// One instantiation of the weight-gradient GEMM (UT = hidden units per workgroup tile).
template <bool FRAG, int UT, int CT>
static hipError_t launch_dw_ttt(const uint16_t* Act, const uint16_t* Hin, const int32_t* offsets,
                               const int32_t* tok, const int32_t* border, const uint16_t* zero_row, int N,
                               int Bs, int d, float* dW, int slot, hipStream_t st, const DwPiece* pieces,
                               int nblocks, float* stage) {
  const int nct = (d + CT - 1) / CT;
  int gx;
  if (nct % 8 == 0) gx = nct * N;
  else if (8 % nct == 0) gx = 8 * ((N + 8 / nct - 1) / (8 / nct));
  else gx = nct * N;
  const dim3 grid(gx, (Bs + UT - 1) / UT);
  const int dw_smem = DW_SLOTS * ((CT / 256) * DW_HALF_BYTES + DW_KT * UT * 2);
  static bool attr_set = false;
  if (!attr_set) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kq_gemm_kernel<FRAG, UT, CT>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, dw_smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  {
    ScopedKernelTimer tm(slot, st);
    kq_gemm_kernel<FRAG, UT, CT><<<grid, CT, dw_smem, st>>>(Act, Hin, offsets, tok, border, zero_row, N, Bs, d, dW,
                                                         pieces, nblocks, stage);
  }
  return hipGetLastError();
}

// 512-column workgroups where each CU still gets at least four of them one after the other (with
// fewer, the uneven last round costs more than the shared hidden-unit copies save: measured on the
// skewed OPT-1.3B-like shape), 256-column ones otherwise.
template <bool FRAG, int UT>
static hipError_t launch_dw_tt(const uint16_t* Act, const uint16_t* Hin, const int32_t* offsets,
                               const int32_t* tok, const int32_t* border, const uint16_t* zero_row, int N,
                               int Bs, int d, float* dW, int slot, hipStream_t st, const DwPiece* pieces,
                               int nblocks, float* stage) {
  if (d % 512 == 0 && (int64_t)(d / 512) * N >= 1024)
    return launch_dw_ttt<FRAG, UT, 512>(Act, Hin, offsets, tok, border, zero_row, N, Bs, d, dW, slot, st, pieces,
                                        nblocks, stage);
  return launch_dw_ttt<FRAG, UT, 256>(Act, Hin, offsets, tok, border, zero_row, N, Bs, d, dW, slot, st, pieces,
                                      nblocks, stage);
}

// dW[b][u][c] = sum_{q in bucket b} Hin[q][u] * Act[tok[q]][c] for N buckets of Bs units and d
// columns (the narrow-block weight-gradient GEMM; also run with a 32-wide side for the adapter
// gradients of the low-rank variant).
template <bool FRAG>
static hipError_t launch_dw_t(const uint16_t* Act, const uint16_t* Hin, const int32_t* offsets,
                              const int32_t* tok, const int32_t* border, const uint16_t* zero_row, int N,
                              int Bs, int d, float* dW, int slot, hipStream_t st,
                              const DwPiece* pieces = nullptr, int nblocks = 0, float* stage = nullptr) {
  return Bs <= 64 ? launch_dw_tt<FRAG, 64>(Act, Hin, offsets, tok, border, zero_row, N, Bs, d, dW, slot, st, pieces,
                                           nblocks, stage)
                  : launch_dw_tt<FRAG, 128>(Act, Hin, offsets, tok, border, zero_row, N, Bs, d, dW, slot, st,
                                            pieces, nblocks, stage);
}

hipError_t launch_dw(const uint16_t* Act, const uint16_t* Hin, bool hin_frag, const int32_t* offsets,
                     const int32_t* tok, const int32_t* border, const uint16_t* zero_row, int N, int Bs, int d,
                     float* dW, int slot, hipStream_t st) {
  return hin_frag ? launch_dw_t<true>(Act, Hin, offsets, tok, border, zero_row, N, Bs, d, dW, slot, st)
                  : launch_dw_t<false>(Act, Hin, offsets, tok, border, zero_row, N, Bs, d, dW, slot, st);
}

hipError_t launch_dw_pieces(const uint16_t* Act, const uint16_t* Hin, bool hin_frag, const Schedule& sc, int N,
                            int Bs, int d, float* dW, float* stage, int slot, hipStream_t st) {
  ScopedKernelTimer tm(slot, st);   // (covers the GEMM and the sum of the staged pieces)
  const hipError_t e =
      hin_frag ? launch_dw_t<true>(Act, Hin, nullptr, sc.tok, nullptr, sc.zero_row, sc.dw_cap, Bs, d, dW, -1, st,
                                   sc.dw_pieces, N, stage)
               : launch_dw_t<false>(Act, Hin, nullptr, sc.tok, nullptr, sc.zero_row, sc.dw_cap, Bs, d, dW, -1, st,
                                    sc.dw_pieces, N, stage);
  if (e != hipSuccess) return e;
  dw_reduce_kernel<<<1024, 256, 0, st>>>(dW, stage, sc.dw_xlist, Bs, d);
  return hipGetLastError();
}

static WideArgs wide_args(const spt_shape_t& s, const int32_t* offsets, const Schedule& sc) {
  WideArgs a = {};
  a.offsets = offsets;
  a.kd_count = sc.kd_count;
  a.kd_list = sc.kd_list;
  a.cap = sc.kd_cap;
  a.tok = sc.tok;
  a.border = sc.border;
  a.zero_row = sc.zero_row;
  a.N = s.N; a.Bs = s.Bs; a.d = s.d;
  return a;
}

hipError_t run_fwd(const spt_shape_t& s, const void* X, const void* W1, const void* W2,
                   const int32_t* offsets, const int32_t* perm, const int32_t* inv, void* Y,
                   void* Hsave, const FwdWorkspace& w, hipStream_t st, const Schedule* prebuilt) {
  const Schedule& sc = prebuilt ? *prebuilt : w.sched;
  hipError_t e = prebuilt ? hipSuccess : run_plan(s, offsets, perm, sc, st);
  if (e != hipSuccess) return e;
  auto x = static_cast<const uint16_t*>(X);
  auto w1 = static_cast<const uint16_t*>(W1);
  auto w2 = static_cast<const uint16_t*>(W2);
  auto hs = static_cast<uint16_t*>(Hsave);
  if (use_narrow(s)) {
    {
      ScopedKernelTimer tm(kSlotUp, st);
      e = launch_up<0>(s, w1, x, offsets, sc, hs, w.Hact, nullptr, st);
    }
    if (e != hipSuccess) return e;
    ScopedKernelTimer tm(kSlotDown, st);
    return launch_scatter(s, plan_scatter(s), w.Hact, w2, sc.rstart, sc.tok,
                          static_cast<uint16_t*>(Y), nullptr, st);
  }
  WideArgs a = wide_args(s, offsets, sc);
  a.A = w1; a.B = x; a.Hsave = hs; a.Hact = w.Hact;
  {
    ScopedKernelTimer tm(kSlotUp, st);
    e = launch_wide(kWideUp, s, a, st);
  }
  if (e != hipSuccess) return e;
  a.A = w2; a.B = w.Hact; a.part = w.part;
  {
    ScopedKernelTimer tm(kSlotDown, st);
    e = launch_wide(kWidePart, s, a, st);
  }
  if (e != hipSuccess) return e;
  return run_combine(s, w.part, inv, Y, 0, s.d, (size_t)s.d, (size_t)TILE, kSlotCombineY, st);
}

hipError_t run_bwd(const spt_shape_t& s, const void* X, const void* W1, const void* W2,
                   const void* dY, const int32_t* offsets, const int32_t* perm,
                   const int32_t* inv, const void* Hsave, void* dX, float* dW1, float* dW2,
                   const BwdWorkspace& w, hipStream_t st, const Schedule* prebuilt) {
  const Schedule& sc = prebuilt ? *prebuilt : w.sched;
  hipError_t e = prebuilt ? hipSuccess : run_plan(s, offsets, perm, sc, st);
  if (e != hipSuccess) return e;
  auto x = static_cast<const uint16_t*>(X);
  auto w1 = static_cast<const uint16_t*>(W1);
  auto w2 = static_cast<const uint16_t*>(W2);
  auto dy = static_cast<const uint16_t*>(dY);
  auto hs = const_cast<uint16_t*>(static_cast<const uint16_t*>(Hsave));
  if (!use_narrow(s)) {
    WideArgs a = wide_args(s, offsets, sc);
    a.A = w2; a.B = dy; a.Hsave = hs; a.Hact = w.Hact; a.dHpre = w.dHpre;
    {
      ScopedKernelTimer tm(kSlotDH, st);
      e = launch_wide(kWideDH, s, a, st);
    }
    if (e != hipSuccess) return e;
    a.A = dy; a.B = w.Hact; a.dW = dW2;
    {
      ScopedKernelTimer tm(kSlotDW2, st);
      e = launch_wide(kWideDW, s, a, st);
    }
    if (e != hipSuccess) return e;
    a.A = x; a.B = w.dHpre; a.dW = dW1;
    {
      ScopedKernelTimer tm(kSlotDW1, st);
      e = launch_wide(kWideDW, s, a, st);
    }
    if (e != hipSuccess) return e;
    a.A = w1; a.B = w.dHpre; a.part = w.part;
    {
      ScopedKernelTimer tm(kSlotDXPart, st);
      e = launch_wide(kWidePart, s, a, st);
    }
    if (e != hipSuccess) return e;
    return run_combine(s, w.part, inv, dX, 0, s.d, (size_t)s.d, (size_t)TILE, kSlotCombineDX, st);
  }
  {
    ScopedKernelTimer tm(kSlotDH, st);
    e = launch_up<1>(s, w2, dy, offsets, sc, hs, w.Hact, w.dHpre, st);
  }
  if (e != hipSuccess) return e;
  {
    ScopedKernelTimer tm(kSlotDXPart, st);
    e = launch_scatter(s, plan_scatter(s), w.dHpre, w1, sc.rstart, sc.tok, static_cast<uint16_t*>(dX),
                       nullptr, st);
  }
  if (e != hipSuccess) return e;
  e = launch_dw_pieces(dy, w.Hact, true, sc, s.N, s.Bs, s.d, dW2, w.dw_stage, kSlotDW2, st);
  if (e != hipSuccess) return e;
  return launch_dw_pieces(x, w.dHpre, true, sc, s.N, s.Bs, s.d, dW1, w.dw_stage, kSlotDW1, st);
}

// ------------------------------------------------------------------------------------------
// Low-rank adapted path (section 2.2 on top of section 4.2).
constexpr size_t kLoraPiece = 512;
static size_t lora_piece_rows(const spt_shape_t& s) {
  size_t piece = kLoraPiece;
  while ((size_t)s.T * s.k / piece + s.N > 1024) piece *= 2;
  return piece;
}
static size_t lora_chunk_tokens(const spt_shape_t& s) {
  // chunks of the token axis for the K = T adapter gradients: at least 512 tokens, at most 1024 chunks
  size_t c = 512;
  while (((size_t)s.T + c - 1) / c > 1024) c *= 2;
  return c;
}

LoraWorkspace plan_lora(const spt_shape_t& s, void* ws, bool backward) {
  const size_t P = (size_t)s.T * s.k, D = (size_t)s.N * s.Bs, T = s.T, d = s.d;
  char* p = static_cast<char*>(ws);
  size_t o = 0;
  LoraWorkspace w = {};
  auto take = [&](size_t bytes) { void* r = p + o; o += align256(bytes); return r; };
  if (backward) { w.bwd = plan_bwd(s, ws, false); o = w.bwd.bytes; }
  else          { w.fwd = plan_fwd(s, ws); o = w.fwd.bytes; }
  w.A1T = static_cast<uint16_t*>(take(32 * d * 2));
  w.C1T = static_cast<uint16_t*>(take(D * 64 * 2));
  w.C1P = static_cast<uint16_t*>(take(32 * D * 2));
  w.B2T = static_cast<uint16_t*>(take(32 * D * 2));
  w.B2P = static_cast<uint16_t*>(take(D * 64 * 2));
  w.C2P = static_cast<uint16_t*>(take(32 * d * 2));
  w.A1P = static_cast<uint16_t*>(take(d * 32 * 2));
  w.C2T = static_cast<uint16_t*>(take(d * 32 * 2));
  w.Z = static_cast<uint16_t*>(take(T * d * 2));
  w.Upad = static_cast<uint16_t*>(take(T * 64 * 2));
  w.Gpad = static_cast<uint16_t*>(take(T * 64 * 2));
  w.Sb = static_cast<uint16_t*>(take(T * 32 * 2));
  w.Sp = static_cast<float*>(take(P * 32 * 4));
  w.Sf = static_cast<float*>(take(T * 32 * 4));
  if (backward) {
    const size_t chunk = lora_chunk_tokens(s), nc = (T + chunk - 1) / chunk;
    // pieces of at most kLoraPiece rows; at most 1024 of them (the dW kernel's bucket limit)
    w.max_pieces = (int)(P / lora_piece_rows(s) + s.N);
    w.gpad = static_cast<float*>(take((size_t)w.max_pieces * s.Bs * 64 * 4));
    w.p_first = static_cast<int32_t*>(take((size_t)(s.N + 1) * 4));
    w.p_off = static_cast<int32_t*>(take((size_t)(w.max_pieces + 1) * 4));
    w.p_id = static_cast<int32_t*>(take((size_t)w.max_pieces * 4));
    w.gchunks = static_cast<float*>(take(nc * 32 * d * 4));
    w.c_off = static_cast<int32_t*>(take((nc + 1) * 4));
    w.c_tok = static_cast<int32_t*>(take(T * 4));
    w.c_border = static_cast<int32_t*>(take(nc * 4));
  }
  w.bytes = o;
  return w;
}

hipError_t run_lora_fwd(const spt_shape_t& s, int r, const void* X, const void* W1, const void* W2,
                        const void* A1, const void* C1, const void* B2, const void* C2,
                        const int32_t* offsets, const int32_t* perm, const int32_t* inv, void* Y,
                        void* Hsave, const LoraWorkspace& w, hipStream_t st) {
  const int D = s.N * s.Bs, P = s.T * s.k;
  auto x = static_cast<const uint16_t*>(X);
  auto hs = static_cast<uint16_t*>(Hsave);
  hipError_t e = run_plan(s, offsets, perm, w.fwd.sched, st);
  if (e != hipSuccess) return e;
  {
    ScopedKernelTimer tm(kSlotLoraSmall, st);
    const uint16_t *a1 = static_cast<const uint16_t*>(A1), *c1 = static_cast<const uint16_t*>(C1);
    const uint16_t *b2 = static_cast<const uint16_t*>(B2), *c2 = static_cast<const uint16_t*>(C2);
    PadJobs jobs = {};
    jobs.job[0] = PadJob{a1, s.d, r, 1, 0, w.A1T, 32, s.d};   // A1^T      [32][d]
    jobs.job[1] = PadJob{c1, r, D, 1, 1, w.C1T, D, 64};       // C1^T twice [D][64]
    jobs.job[2] = PadJob{b2, D, r, 1, 0, w.B2T, 32, D};       // B2^T      [32][D]
    jobs.job[3] = PadJob{c2, r, s.d, 1, 0, w.C2T, s.d, 32};   // C2^T      [d][32]
    if ((e = lora_pad(jobs, 4, st)) != hipSuccess) return e;
    if ((e = lora_proj(x, w.A1T, s.T, s.d, w.Upad, st)) != hipSuccess) return e;
  }
  const bool narrow = use_narrow(s);
  if (narrow) {
    ScopedKernelTimer tm(kSlotUp, st);
    e = launch_up<0>(s, static_cast<const uint16_t*>(W1), x, offsets, w.fwd.sched, hs, w.fwd.Hact, nullptr, st,
                     w.Upad, w.C1T);
    if (e != hipSuccess) return e;
  } else {
    WideArgs a = wide_args(s, offsets, w.fwd.sched);
    a.A = W1; a.B = x; a.Hsave = hs; a.Hact = w.fwd.Hact; a.Xe = w.Upad; a.We = w.C1T;
    {
      ScopedKernelTimer tm(kSlotUp, st);
      e = launch_wide(kWideUp, s, a, st);
    }
    if (e != hipSuccess) return e;
    a.A = W2; a.B = w.fwd.Hact; a.part = w.fwd.part; a.Xe = nullptr; a.We = nullptr;
    {
      ScopedKernelTimer tm(kSlotDown, st);
      e = launch_wide(kWidePart, s, a, st);
    }
    if (e != hipSuccess) return e;
  }
  {
    // V[t] = sum_b B2_b^T h_b(t);  Z = V C2, the low-rank row the write-back adds per token
    ScopedKernelTimer tm(kSlotLoraSmall, st);
    if ((e = lora_pair_gemm(w.fwd.Hact, narrow, w.B2T, offsets, s.N, s.Bs, P, 2, w.Sp, st)) != hipSuccess) return e;
    if ((e = lora_token_sum(w.Sp, inv, s.T, s.k, w.Sf, nullptr, st)) != hipSuccess) return e;
    if ((e = lora_expand(w.Sf, w.C2T, s.T, s.d, w.Z, st)) != hipSuccess) return e;
  }
  if (!narrow) return run_combine(s, w.fwd.part, inv, Y, 0, s.d, (size_t)s.d, (size_t)TILE, kSlotCombineY, st, w.Z);
  ScopedKernelTimer tm(kSlotDown, st);
  return launch_scatter(s, plan_scatter(s), w.fwd.Hact, static_cast<const uint16_t*>(W2), w.fwd.sched.rstart,
                        w.fwd.sched.tok, static_cast<uint16_t*>(Y), w.Z, st);
}

hipError_t run_lora_bwd(const spt_shape_t& s, int r, const void* X, const void* W1, const void* W2,
                        const void* A1, const void* C1, const void* B2, const void* C2, const void* dY,
                        const int32_t* offsets, const int32_t* perm, const int32_t* inv,
                        const void* Hsave, void* dX, float* dA1, float* dC1, float* dB2, float* dC2,
                        const LoraWorkspace& w, hipStream_t st) {
  const int D = s.N * s.Bs, P = s.T * s.k;
  auto x = static_cast<const uint16_t*>(X);
  auto dy = static_cast<const uint16_t*>(dY);
  auto hs = const_cast<uint16_t*>(static_cast<const uint16_t*>(Hsave));
  const Schedule& sc = w.bwd.sched;
  hipError_t e = run_plan(s, offsets, perm, sc, st);
  if (e != hipSuccess) return e;
  const int chunk = (int)lora_chunk_tokens(s), nc = (s.T + chunk - 1) / chunk;
  {
    ScopedKernelTimer tm(kSlotLoraSmall, st);
    const uint16_t *a1 = static_cast<const uint16_t*>(A1), *c1 = static_cast<const uint16_t*>(C1);
    const uint16_t *b2 = static_cast<const uint16_t*>(B2), *c2 = static_cast<const uint16_t*>(C2);
    PadJobs jobs = {};
    jobs.job[0] = PadJob{a1, s.d, r, 1, 0, w.A1T, 32, s.d};   // A1^T       [32][d]
    jobs.job[1] = PadJob{a1, s.d, r, 0, 0, w.A1P, s.d, 32};   // A1         [d][32]
    jobs.job[2] = PadJob{c1, r, D, 0, 0, w.C1P, 32, D};       // C1         [32][D]
    jobs.job[3] = PadJob{b2, D, r, 1, 0, w.B2T, 32, D};       // B2^T       [32][D]
    jobs.job[4] = PadJob{b2, D, r, 0, 1, w.B2P, D, 64};       // B2 twice   [D][64]
    jobs.job[5] = PadJob{c2, r, s.d, 0, 0, w.C2P, 32, s.d};   // C2         [32][d]
    if ((e = lora_pad(jobs, 6, st)) != hipSuccess) return e;
    if ((e = lora_proj(x, w.A1T, s.T, s.d, w.Upad, st)) != hipSuccess) return e;   // U = X A1
    if ((e = lora_proj(dy, w.C2P, s.T, s.d, w.Gpad, st)) != hipSuccess) return e;  // G = dY C2^T
    if ((e = lora_chunks(s.T, chunk, nc, w.c_off, w.c_tok, w.c_border, st)) != hipSuccess) return e;
    if ((e = lora_pieces(offsets, s.N, (int)lora_piece_rows(s), w.max_pieces, w.p_first, w.p_off, w.p_id,
                         st)) != hipSuccess) return e;
  }
  const bool narrow = use_narrow(s);
  if (narrow) {
    // dH = dY W2_b^T + G B2_b^T; dHpre and Hact go to the workspace
    ScopedKernelTimer tm(kSlotDH, st);
    e = launch_up<1>(s, static_cast<const uint16_t*>(W2), dy, offsets, sc, hs, w.bwd.Hact, w.bwd.dHpre, st,
                     w.Gpad, w.B2P);
    if (e != hipSuccess) return e;
  } else {
    WideArgs a = wide_args(s, offsets, sc);
    a.A = W2; a.B = dy; a.Hsave = hs; a.Hact = w.bwd.Hact; a.dHpre = w.bwd.dHpre; a.Xe = w.Gpad; a.We = w.B2P;
    {
      ScopedKernelTimer tm(kSlotDH, st);
      e = launch_wide(kWideDH, s, a, st);
    }
    if (e != hipSuccess) return e;
    a.A = W1; a.B = w.bwd.dHpre; a.part = w.bwd.part; a.Xe = nullptr; a.We = nullptr;
    {
      ScopedKernelTimer tm(kSlotDXPart, st);
      e = launch_wide(kWidePart, s, a, st);
    }
    if (e != hipSuccess) return e;
  }
  {
    // R[t] = sum_b C1_b dhpre_b(t)
    ScopedKernelTimer tm(kSlotLoraSmall, st);
    if ((e = lora_pair_gemm(w.bwd.dHpre, narrow, w.C1P, offsets, s.N, s.Bs, P, 2, w.Sp, st)) != hipSuccess) return e;
    if ((e = lora_token_sum(w.Sp, inv, s.T, s.k, w.Sf, w.Sb, st)) != hipSuccess) return e;
    if ((e = lora_expand(w.Sf, w.A1P, s.T, s.d, w.Z, st)) != hipSuccess) return e;  // Z = R A1^T
  }
  // dX = sum_b dhpre_b W1_b + R A1^T
  if (narrow) {
    ScopedKernelTimer tm(kSlotDXPart, st);
    e = launch_scatter(s, plan_scatter(s), w.bwd.dHpre, static_cast<const uint16_t*>(W1), sc.rstart, sc.tok,
                       static_cast<uint16_t*>(dX), w.Z, st);
  } else {
    e = run_combine(s, w.bwd.part, inv, dX, 0, s.d, (size_t)s.d, (size_t)TILE, kSlotCombineDX, st, w.Z);
  }
  if (e != hipSuccess) return e;
  // dA1[i][rho] = sum_t X[t][i] R[t][rho]: the dW GEMM over token chunks, then a sum over chunks
  e = launch_dw(x, w.Sb, false, w.c_off, w.c_tok, w.c_border, sc.zero_row, nc, 32, s.d, w.gchunks, kSlotLoraGrad, st);
  if (e != hipSuccess) return e;
  if ((e = lora_reduce(w.gchunks, nc, 32, s.d, true, false, dA1, s.d, r, st)) != hipSuccess) return e;
  // dC1[rho][unit] = sum_{q in b} U[tok q][rho] dHpre[q][u]
  // (U as its two bf16 parts, 64 columns: the two products are added when the result is unpacked)
  // per piece of a bucket, then summed over the bucket's pieces in order
  e = launch_dw(w.Upad, w.bwd.dHpre, narrow, w.p_off, sc.tok, w.p_id, sc.zero_row, w.max_pieces, s.Bs, 64, w.gpad,
                kSlotLoraGrad, st);
  if (e != hipSuccess) return e;
  if ((e = lora_reduce_pieces(w.gpad, w.p_first, s.N, s.Bs, r, true, dC1, st)) != hipSuccess) return e;
  // dB2[unit][rho] = sum_{q in b} Hact[q][u] G[tok q][rho]
  e = launch_dw(w.Gpad, w.bwd.Hact, narrow, w.p_off, sc.tok, w.p_id, sc.zero_row, w.max_pieces, s.Bs, 64, w.gpad,
                kSlotLoraGrad, st);
  if (e != hipSuccess) return e;
  if ((e = lora_reduce_pieces(w.gpad, w.p_first, s.N, s.Bs, r, false, dB2, st)) != hipSuccess) return e;
  // V[t] = sum_b B2_b^T h_b(t);  dC2[rho][c] = sum_t V[t][rho] dY[t][c]
  {
    ScopedKernelTimer tm(kSlotLoraSmall, st);
    if ((e = lora_pair_gemm(w.bwd.Hact, narrow, w.B2T, offsets, s.N, s.Bs, P, 2, w.Sp, st)) != hipSuccess) return e;
    if ((e = lora_token_sum(w.Sp, inv, s.T, s.k, nullptr, w.Sb, st)) != hipSuccess) return e;
  }
  e = launch_dw(dy, w.Sb, false, w.c_off, w.c_tok, w.c_border, sc.zero_row, nc, 32, s.d, w.gchunks, kSlotLoraGrad, st);
  if (e != hipSuccess) return e;
  return lora_reduce(w.gchunks, nc, 32, s.d, false, false, dC2, r, s.d, st);
}

}  // namespace spt
