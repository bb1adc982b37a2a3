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
// Operands.  The weight slice (Bs x 64 columns, hidden-unit major as stored) travels global ->
// registers -> LDS stage and is turned into K-contiguous MFMA fragments by ds_read_b64_tr_b16;
// the fragments of a run live in registers, so a stage is free again as soon as they are read.
// Hin is stored in fragment order (ffn_common.hpp): the 16 bytes per K-step of 32 consecutive
// rows are one contiguous kilobyte, which goes straight from global memory into the lanes that
// own the rows.  Both are requested several runs ahead of their use.
// Every load is an ordinary load, so all vmcnt bookkeeping is the compiler's (asynchronous
// global -> LDS copies would be invisible to it, and it would then wait too long for the loads
// it can see).  Four wavefronts, one 32-row tile each; a run longer than 128 rows takes more
// passes over the same register-resident weight fragments.
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

__device__ __forceinline__ void sc_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

// Run table.  For token range r (tokens r R .. r R + R - 1) and bucket b the rows of the bucket
// that belong to the range are one contiguous run of sorted positions (inside a bucket the token
// ids ascend): [starts[r][b], starts[r+1][b]), a dense table the schedule kernel fills.  One
// wavefront per range turns its two table rows into the list of the range's NON-EMPTY runs, in
// ascending block order and cut into pieces of at most SC_RUN rows (one pass of the GEMM
// kernel's four row tiles), as (block, first, end, 0) records, and their count.  A range has at
// most N + R k / SC_RUN records.
constexpr int SC_RUN = 128;
struct RunRec { int32_t b, lo, hi, pad; };

__global__ __launch_bounds__(64) void scatter_runs_kernel(const int32_t* __restrict__ starts, int N, int cap,
                                                          RunRec* __restrict__ runs,
                                                          int32_t* __restrict__ nruns) {
  const int r = blockIdx.x, lane = threadIdx.x;
  const int32_t* s0 = starts + (size_t)r * N;
  const int32_t* s1 = s0 + N;
  RunRec* list = runs + (size_t)r * cap;
  int count = 0;
  for (int b0 = 0; b0 < N; b0 += 64) {
    const int b = b0 + lane;
    const int first = (b < N) ? s0[b] : 0, end = (b < N) ? s1[b] : 0;
    const int pieces = (end - first + SC_RUN - 1) / SC_RUN;
    int incl = pieces;  // inclusive scan over the wavefront
#pragma unroll
    for (int sft = 1; sft < 64; sft <<= 1) {
      const int up = __shfl_up(incl, sft);
      if (lane >= sft) incl += up;
    }
    int at = count + incl - pieces;
    for (int p = 0; p < pieces; ++p, ++at)
      if (at < cap) list[at] = RunRec{b, first + p * SC_RUN, min(first + (p + 1) * SC_RUN, end), 0};
    count += __shfl(incl, 63);
  }
  if (lane == 0) nruns[r] = count < cap ? count : cap;
}

// KS = Bs / 16 K-steps per block.  A workgroup owns R tokens x 64 output columns; a run (at most
// 128 rows) is four 32-row tiles, one per wavefront, by two 32-column tiles.
//
// The loop over a range's runs is software-pipelined so that the operands of a run are in
// registers when its turn comes.  The slab rows of a run (the running sums of its tokens, 64
// bytes per lane and column tile) are read straight INTO the accumulators, the matrix cores add
// the run's products on top, and the accumulators go back to the same place: the
// read-modify-write costs no vector instruction.  Consecutive runs update the same token rows (a
// token often activates consecutive blocks), so one barrier per iteration separates them.
// Iteration j:
//     barrier               run j-1 is in the slab, weight slice j+1 visible, stage j free
//     read tiles 0 and 1 of run j's slab rows -> accumulators
//     stage weight slice j+2, request slice j+4, token ids, Hin rows of run j+2
//     MFMAs of tile 0, write tile 0     (tile 1's slab values arrive meanwhile)
//     MFMAs of tile 1, write tile 1     (tile 0's write completes meanwhile)
// with the fragment reads of run j+1 spread behind the MFMAs.  Lanes past the end of a run skip
// the slab accesses by EXEC mask only, so the loop body has no branch; whatever their
// accumulators hold stays in their own lane (an MFMA output column depends on its own B-operand
// column only).
// Measured on the 7B-like shape, in the order built: slab update by vector adds, one run behind
// the MFMAs, 0.67 ms; slab rows through the accumulators, one K loop over both tiles 0.645; the K
// loop in two halves per tile 0.600; tile after tile, as here, 0.585; a second barrier in the
// middle so that tile 0 of the next run can be read an iteration ahead 0.62 (the barrier drains
// the LDS queue).  Two wavefronts with two row tiles each (weight fragments read half as often)
// took 0.91 ms, eight with one column tile each (Hin rows loaded twice) 0.71 ms.
constexpr int SC_C = 64;                     // output columns per workgroup
constexpr int SC_STRIDE = SC_C * 4 + SC_PAD; // bytes per slab row
constexpr int SC_STAGES = 2;                 // weight-slice stages in LDS

template <int KS>
__global__ __launch_bounds__(SC_THREADS, 1) void ffn_scatter_kernel(
    const uint16_t* __restrict__ Hin, const uint16_t* __restrict__ W, const RunRec* __restrict__ runs,
    const int32_t* __restrict__ nruns, const int32_t* __restrict__ tok, int N, int d, int T, int R,
    int nr, int nslab, int cap, uint16_t* __restrict__ out, const uint16_t* __restrict__ Z) {
  constexpr int Bs = KS * 16;
  constexpr int THREADS = SC_THREADS;
  constexpr int NWAVES = THREADS / 64;
  constexpr int PIECES = 2 * KS;               // kilobytes of a weight slice
  constexpr int NW = (PIECES + NWAVES - 1) / NWAVES;   // 16-byte pieces of a weight slice per lane
  constexpr int STAGE_BYTES = Bs * 128;
  extern __shared__ uint4 sc_smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int rtile = wave;                      // this wavefront's 32-row tile of a run
  const int i = lane & 31, h = lane >> 5;

  // Work item.  With a multiple of 8 slabs an XCD (workgroup id mod 8) keeps to its own slabs
  // and the workgroups it runs together are token ranges x up to 8 slabs (all of its slabs at
  // d = 4096: every run of Hin rows is then fetched once per XCD): per block they want a few weight
  // slices and a few runs of Hin rows, which its L2 serves to all of them.
  int r, slab;
  if (nslab % 8 == 0) {
    const int spx = nslab >> 3, x = blockIdx.x & 7, j = blockIdx.x >> 3;
    const int inner = spx < 8 ? spx : 8;       // slabs that run side by side
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

  char* slab_lds = reinterpret_cast<char*>(sc_smem);           // R + 1 rows: the last one is the dummy
  const int ring_off = (R + 1) * SC_STRIDE;
  char* ring = slab_lds + ring_off;

  typedef const __attribute__((address_space(4))) RunRec* const_run_ptr;
  const const_run_ptr rl = (const_run_ptr)(uintptr_t)(runs + (size_t)r * cap);
  const int M = __builtin_amdgcn_readfirstlane(nruns[r]);
  struct Run { int b, lo, hi; bool real; };
  auto run_at = [&](int j) {  // wave-uniform scalar load; past the end: the last run again, marked unreal
    const int jj = j < M ? j : (M > 0 ? M - 1 : 0);
    return Run{rl[jj].b, rl[jj].lo, rl[jj].hi, j < M};
  };

  // weight slice: piece j of this lane is 16 bytes of stage row 8 (wave NW + j) + lane / 8 (a stage
  // row = 128 bytes = one hidden unit x 64 columns), physical 16-byte slot lane % 8 = logical ^
  // (((row >> 1) & 1) << 2)
  struct Slice { u32x4 v[NW]; };
  // (where the pieces do not divide evenly among the wavefronts, the surplus ones repeat a
  // piece: same bytes to the same place, and no branch in the loop)
  int w_off[NW], w_piece[NW];
#pragma unroll
  for (int j = 0; j < NW; ++j) {
    w_piece[j] = (wave * NW + j) % PIECES;
    const int unit = 8 * w_piece[j] + (lane >> 3);
    const int ch = (lane & 7) ^ (((unit >> 1) & 1) << 2);
    w_off[j] = unit * d + c0 + ch * 8;
  }
  auto load_w = [&](Slice& w, int b) {
    const uint16_t* wb = W + (size_t)b * Bs * d;
#pragma unroll
    for (int j = 0; j < NW; ++j) w.v[j] = *reinterpret_cast<const u32x4*>(wb + w_off[j]);
  };
  auto store_w = [&](const Slice& w, int stage) {
    char* st = ring + stage * STAGE_BYTES + lane * 16;
#pragma unroll
    for (int j = 0; j < NW; ++j) *reinterpret_cast<u32x4*>(st + w_piece[j] * 1024) = w.v[j];
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
  // end read its first row
  struct RowTile { bf16x8 hb[KS]; bool live; };
  auto row_of = [&](bool& live, const Run& run) {
    const int q = run.lo + rtile * 32 + i;
    live = q < run.hi && run.real;
    return q < run.hi ? q : run.lo;
  };
  auto load_rows = [&](RowTile& rt, const Run& run) {
    const int qq = row_of(rt.live, run);
    const uint4* src = reinterpret_cast<const uint4*>(Hin + hfrag_off(qq, 8 * h, Bs));
#pragma unroll
    for (int s = 0; s < KS; ++s) rt.hb[s] = as_bf16x8(src[64 * s]);   // K-step s: 1 KiB further
  };
  // the lane's 64 bytes of column tile 0 in its token's slab row (tile 1: 128 bytes further)
  auto slab_ptr = [&](bool live, int token) {
    return reinterpret_cast<f32x4*>(slab_lds + (live ? token - t0 : R) * SC_STRIDE + 64 * h);
  };
  auto slab_read = [&](f32x16& a, const f32x4* p) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const f32x4 o = p[c];
      a[4 * c] = o[0]; a[4 * c + 1] = o[1]; a[4 * c + 2] = o[2]; a[4 * c + 3] = o[3];
    }
  };
  auto slab_write = [&](f32x4* p, const f32x16& a) {
#pragma unroll
    for (int c = 0; c < 4; ++c) p[c] = f32x4{a[4 * c], a[4 * c + 1], a[4 * c + 2], a[4 * c + 3]};
  };
  // ---- prologue: request the first operands, clear the slab while they fly, stage slices 0 and
  // 1 and read run 0's fragments.  (Every token activates k >= 1 blocks, so a range always has
  // runs; M = 0 means a caller's table that lists nothing for these tokens: zeros.)
  if (M == 0) {
    for (int it = tid; it < rows * (SC_C / 8); it += THREADS) {
      const size_t o = (size_t)(t0 + it / (SC_C / 8)) * d + c0 + (it % (SC_C / 8)) * 8;
      *reinterpret_cast<uint4*>(out + o) = Z ? *reinterpret_cast<const uint4*>(Z + o) : make_uint4(0u, 0u, 0u, 0u);
    }
    return;
  }
  // (requests past the last run repeat it -- run_at clamps -- into registers nobody uses any
  // more: the loop has no branch around a load, which keeps the compiler's vmcnt waits exact)
  Run q0 = run_at(0), q1 = run_at(1), q2 = run_at(2), q3 = run_at(3), q4 = run_at(4);
  Slice wbuf[2];
  RowTile hbuf[2];
  bf16x8 af[2][2][KS];
  f32x16 acc0, acc1;      // column tiles 0 and 1
  // Token ids of the lane's rows: both halves of an unrolled pair of iterations request theirs in
  // the first half (tok_next[0] for the run two iterations on, tok_next[1] for the one after it),
  // and the second half works on a copy taken a whole pair later.  A loop-carried copy of a loaded
  // register makes the compiler wait for that load where the copy is made; this way every such
  // wait is for a request at least an iteration old.  The prologue issues its requests in the
  // order of a pair of iterations (ids, slice, rows, slice, rows), so the compiler's count of
  // outstanding loads is the same on both ways into the loop and its waits come out exact.
  int tok_next[2], tok_second = 0;
  {
    Slice w0, w1;
    load_w(w0, q0.b);
    load_w(w1, q1.b);
    bool unused;
    tok_next[0] = tok[row_of(unused, q0)];
    tok_next[1] = tok[row_of(unused, q1)];
    load_w(wbuf[0], q2.b);
    load_rows(hbuf[0], q0);
    load_w(wbuf[1], q3.b);
    load_rows(hbuf[1], q1);
    for (int o = tid * 16; o < (R + 1) * SC_STRIDE; o += THREADS * 16)
      *reinterpret_cast<uint4*>(slab_lds + o) = make_uint4(0u, 0u, 0u, 0u);
    store_w(w0, 0);
    store_w(w1, 1);
  }
#pragma unroll
  for (int v = 0; v < 16; ++v) { acc0[v] = 0.f; acc1[v] = 0.f; }
  sc_barrier();
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int s = 0; s < KS; ++s)
      af[0][t][s] = tr_read_frag(ring + tr_off[t] + s * 2048, ring + tr_off[t] + s * 2048 + 512);

  // ---- iteration j (0 <= j < M, rounded up to a whole pair).  The loop is unrolled by two so that
  // the double-buffer halves (j mod 2) are compile-time constants.  At the top of iteration j:
  // slice j+1 is in stage (j+1) mod 2, slices j+2 and j+3 are in (or on their way into) wbuf, rows
  // j and j+1 in (or on their way into) hbuf, the fragments of run j in af[j mod 2].
  int j = 0;
  int rd_stage = STAGE_BYTES;   // byte offset of the stage iteration j reads fragments from: (j+1) mod 2
  asm volatile("" : "+s"(rd_stage));
  auto iteration = [&](auto tag) {
    constexpr int par = decltype(tag)::value;
    sc_barrier();      // everyone's slab updates (run j-1) and fragment reads (run j) are done, slice j+1 is visible
    const bool live = hbuf[par].live;
    const int token = (par == 0) ? tok_next[0] : tok_second;
    if (par == 0) tok_second = tok_next[1];
    f32x4* sp = slab_ptr(live, token);
    if (live) { slab_read(acc0, sp); slab_read(acc1, sp + 8); }
    // slice j+2 into the stage slice j left (its fragments were read in iteration j-1, before
    // the barrier), then the requests for the token ids of runs j+2 and j+3 (first half only) and
    // for slice j+4 into the registers just read out
    store_w(wbuf[par], par);
    if (par == 0) {
      bool unused;
      tok_next[0] = tok[row_of(unused, q2)];
      tok_next[1] = tok[row_of(unused, q3)];
    }
    load_w(wbuf[par], q4.b);
    // rows of run j+2: requested piece by piece behind tile 1's MFMAs, the last to read run j's
    const int qq = row_of(hbuf[par].live, q2);
    const uint4* src = reinterpret_cast<const uint4*>(Hin + hfrag_off(qq, 8 * h, Bs));
    // (the stage base is kept a run-time value: as a constant it would make all 4 KS fragment
    // addresses loop invariants that are hoisted into registers instead of immediate offsets)
    const char* st = ring + rd_stage;
    rd_stage = STAGE_BYTES - rd_stage;
    __builtin_amdgcn_sched_barrier(0);
    Run qn;
    // tile 0
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[par][0][s], hbuf[par].hb[s], acc0, 0, 0, 0);
      // (the scalar loads of the run record five runs on go out here, behind the wait for the
      // slab values and a whole K loop ahead of the barrier's wait: in front of either one they
      // would show their full latency in every iteration)
      if (s == 0) qn = run_at(j + 5);
      af[par ^ 1][0][s] = tr_read_frag(st + tr_off[0] + s * 2048, st + tr_off[0] + s * 2048 + 512);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (live) slab_write(sp, acc0);
    __builtin_amdgcn_sched_barrier(0);
    // tile 1
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[par][1][s], hbuf[par].hb[s], acc1, 0, 0, 0);
      hbuf[par].hb[s] = as_bf16x8(src[64 * s]);
      af[par ^ 1][1][s] = tr_read_frag(st + tr_off[1] + s * 2048, st + tr_off[1] + s * 2048 + 512);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (live) slab_write(sp + 8, acc1);
    __builtin_amdgcn_sched_barrier(0);
    q0 = q1; q1 = q2; q2 = q3; q3 = q4; q4 = qn;
    ++j;
  };
  // (always whole pairs, one exit: an exit between the halves would share the latch with the
  // way round, and the compiler would size the waits there for the shorter of the two.  The
  // iteration past the last one sees a run without rows: it updates nothing.)
  do {
    iteration(std::integral_constant<int, 0>{});
    iteration(std::integral_constant<int, 1>{});
  } while (j < M);
  sc_barrier();

  // write the slab out: one rounding to bf16 (+ the low-rank row of the token, if any)
  constexpr int CG = SC_C / 8;  // 16-byte output pieces per row
  if (!Z) {
    for (int it = tid; it < rows * CG; it += THREADS) {
      const f32x4* p = reinterpret_cast<const f32x4*>(slab_lds + (it / CG) * SC_STRIDE + (it % CG) * 32);
      const f32x4 lo4 = p[0], hi4 = p[1];
      *reinterpret_cast<uint4*>(out + (size_t)(t0 + it / CG) * d + c0 + (it % CG) * 8) =
          make_uint4(pack_bf16x2(lo4[0], lo4[1]), pack_bf16x2(lo4[2], lo4[3]), pack_bf16x2(hi4[0], hi4[1]),
                     pack_bf16x2(hi4[2], hi4[3]));
    }
    return;
  }
  constexpr int UN = 4;         // pieces per thread and pass: their low-rank rows are requested together
  for (int it0 = tid; it0 < rows * CG; it0 += THREADS * UN) {
    size_t o[UN];
    uint4 z[UN];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int it = it0 + u * THREADS;
      const int itc = it < rows * CG ? it : it0;   // past the end: the first piece again, not stored
      o[u] = (size_t)(t0 + itc / CG) * d + c0 + (itc % CG) * 8;
      z[u] = *reinterpret_cast<const uint4*>(Z + o[u]);
    }
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int it = it0 + u * THREADS;
      if (it >= rows * CG) break;
      const f32x4* p = reinterpret_cast<const f32x4*>(slab_lds + (it / CG) * SC_STRIDE + (it % CG) * 32);
      f32x4 lo4 = p[0], hi4 = p[1];
      lo4 += f32x4{lo_bf16(z[u].x), hi_bf16(z[u].x), lo_bf16(z[u].y), hi_bf16(z[u].y)};
      hi4 += f32x4{lo_bf16(z[u].z), hi_bf16(z[u].z), lo_bf16(z[u].w), hi_bf16(z[u].w)};
      *reinterpret_cast<uint4*>(out + o[u]) =
          make_uint4(pack_bf16x2(lo4[0], lo4[1]), pack_bf16x2(lo4[2], lo4[3]), pack_bf16x2(hi4[0], hi4[1]),
                     pack_bf16x2(hi4[2], hi4[3]));
    }
  }
}

// ------------------------------------------------------------------------------------------
// host side
ScatterPlan plan_scatter(const spt_shape_t& s) {
  ScatterPlan p;
  const int budget = 160 * 1024 - SC_STAGES * s.Bs * 128 - SC_STRIDE;  // (one slab row is the dummy)
  int rmax = budget / SC_STRIDE;
  if (rmax > 448) rmax = 448;
  p.nslab = s.d / SC_C;
  // ranges: as few as the LDS slab allows, but enough workgroups to occupy the chip when the
  // shape is small (never below 64 tokens per range)
  p.nr = (s.T + rmax - 1) / rmax;
  const int fill = (256 + p.nslab - 1) / p.nslab, cap = (s.T + 63) / 64;
  if (p.nr < fill) p.nr = fill < cap ? fill : (cap > p.nr ? cap : p.nr);
  p.R = (s.T + p.nr - 1) / p.nr;
  p.nr = (s.T + p.R - 1) / p.R;
  p.smem = (p.R + 1) * SC_STRIDE + SC_STAGES * s.Bs * 128;
  p.cap = s.N + (int)(((int64_t)p.R * s.k + SC_RUN - 1) / SC_RUN);
  p.runs_bytes = align256((size_t)p.nr * p.cap * sizeof(RunRec));
  p.counts_bytes = align256((size_t)p.nr * 4);
  p.table_bytes = p.runs_bytes + p.counts_bytes + align256((size_t)(p.nr + 1) * s.N * 4);
  return p;
}

int32_t* scatter_starts(const ScatterPlan& p, int32_t* table) {
  return reinterpret_cast<int32_t*>(reinterpret_cast<char*>(table) + p.runs_bytes + p.counts_bytes);
}

hipError_t run_scatter_ranges(const spt_shape_t& s, const ScatterPlan& p, int32_t* table, hipStream_t st) {
  RunRec* runs = reinterpret_cast<RunRec*>(table);
  int32_t* nruns = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(table) + p.runs_bytes);
  scatter_runs_kernel<<<p.nr, 64, 0, st>>>(scatter_starts(p, table), s.N, p.cap, runs, nruns);
  return hipGetLastError();
}

template <int KS>
static hipError_t launch_scatter_t(const spt_shape_t& s, const ScatterPlan& p, const uint16_t* Hin,
                                   const uint16_t* W, const int32_t* table, const int32_t* tok,
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
    const int spx = p.nslab / 8, inner = spx < 8 ? spx : 8, groups = (spx + inner - 1) / inner;
    grid = 8 * groups * inner * p.nr;
  } else {
    grid = p.nslab * p.nr;
  }
  const RunRec* runs = reinterpret_cast<const RunRec*>(table);
  const int32_t* nruns = reinterpret_cast<const int32_t*>(reinterpret_cast<const char*>(table) + p.runs_bytes);
  ffn_scatter_kernel<KS><<<grid, SC_THREADS, p.smem, st>>>(Hin, W, runs, nruns, tok, s.N, s.d, s.T, p.R, p.nr,
                                                            p.nslab, p.cap, out, Z);
  return hipGetLastError();
}

hipError_t launch_scatter(const spt_shape_t& s, const ScatterPlan& p, const uint16_t* Hin, const uint16_t* W,
                          const int32_t* table, const int32_t* tok, uint16_t* out, const uint16_t* Z,
                          hipStream_t st) {
#define SPT_SC(KS) launch_scatter_t<KS>(s, p, Hin, W, table, tok, out, Z, st)
  switch (s.Bs / 16) {
    case 2: return SPT_SC(2);
    case 4: return SPT_SC(4);
    case 6: return SPT_SC(6);
    case 8: return SPT_SC(8);
    default: return hipErrorInvalidValue;
  }
#undef SPT_SC
}

}  // namespace spt
