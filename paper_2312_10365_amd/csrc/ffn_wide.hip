// Routed FFN, blocks wider than 128 hidden units (the paper's own regime, section 4.2: G = 4 or 8
// groups of D/G units, so a block is 1024-2752 units wide).  Every stage is then a large GEMM
// per bucket and the matrix cores, not the partial-row traffic, bound the path, so all six
// GEMMs of Eq. 4 / Alg. 4 and their derivatives share one mainloop built for reuse:
//
//   C[a][n] = sum_k A[a][k] * B[n][k],  256 x 256 outputs per workgroup, 4 wavefronts 2 x 2,
//   128 x 128 per wavefront (4 x 4 tiles of v_mfma_f32_32x32x16_bf16, 256 accumulator
//   registers), K in stages of 32 through a 5-slot LDS ring (32 KiB per stage, three stages
//   in flight, two resident) filled by global_load_lds_dwordx4 with hand-placed vmcnt waits.
//
//   GEMM                       | A side (MFMA rows)           | B side (MFMA columns)        | K
//   up  (Alg. 4 inner proj.)   | hidden units: rows of W1_b   | bucket rows: gathered X rows | d
//   dH  (backward)             | hidden units: rows of W2_b   | bucket rows: gathered dY     | d
//   down / dX partial rows     | output columns of W2_b / W1_b| bucket rows of H / dHpre     | Bs
//   dW2 / dW1                  | columns of gathered dY / X   | hidden units of H / dHpre    | bucket rows
//
// An operand whose K axis is contiguous in memory (rows of W for up/dH, gathered activation
// rows, rows of H) lands in LDS as 256 rows x 64 bytes and is read with ds_read_b128; one
// whose K axis is the slow one (W for down/dX, everything for dW) lands as 32 K-rows x 512
// bytes exactly as stored and is read with the transposing ds_read_b64_tr_b16.  Either way the
// A side is fed to the MFMA rows through the permutation rho32, so a lane ends up with 16
// CONSECUTIVE A-side indices of one B-side index: every epilogue writes 32- or 64-byte runs.
// Rows or columns past the end of a bucket, of the block or of d are pointed at a valid
// address and never stored; K rows past a bucket's end (dW only) read a row of zeros on the
// B side, so they add nothing.
#include "ffn_common.hpp"
#include "spt_host.hpp"
#include "profile.hpp"

namespace spt {

constexpr int WD = 256;                      // tile edge, both sides
constexpr int WK = 32;                       // K values per stage
constexpr int W_REGION = WD * WK * 2;        // bytes of one operand in a stage (16 KiB)
constexpr int W_STAGE = 2 * W_REGION;        // 32 KiB
constexpr int W_STAGES = 5;
constexpr int W_SMEM = W_STAGES * W_STAGE;   // 160 KiB, the whole LDS of a CU
constexpr int W_RT = 4;                      // row tiles per scheduling group

enum { OP_UP = 0, OP_DH = 1, OP_PART = 2, OP_DW = 3 };

// Identity the compiler cannot see through.  An accumulator value that is used more than once
// would otherwise be copied out of the accumulator registers right after the K loop -- all
// 256 of them at once -- instead of where it is used.
__device__ __forceinline__ float pin_vgpr(float x) {
  asm volatile("" : "+v"(x));
  return x;
}

// One 256 x 256 output tile.  b: block; a0 / n0: first A-side / B-side index; [qb, qe): the K
// range (OP_DW: the bucket's rows) -- for the other GEMMs qe bounds the B-side rows.
template <int OP, int ACT>
__device__ __forceinline__ void wide_tile(const WideArgs& p, uint4* smem, int b, int a0, int n0,
                                          int qb, int qe) {
  constexpr bool A_TR = (OP == OP_PART || OP == OP_DW);
  constexpr bool B_TR = (OP == OP_DW);
  const int Bs = p.Bs, d = p.d;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int i = lane & 31, h = lane >> 5;
  const uint32_t lds0 = (uint32_t)(uintptr_t)smem;
  const uint16_t* __restrict__ Aop = static_cast<const uint16_t*>(p.A);
  const uint16_t* __restrict__ Bop = static_cast<const uint16_t*>(p.B);
  const int a_lim = (OP == OP_UP || OP == OP_DH) ? Bs : d;
  // Low-rank adapters (section 2.2) extend the K = d GEMMs by two stages: 64 more K-values per
  // gathered row (Xe[token][64]) and per hidden unit (We[unit][64]).
  // (Compiled in only when bit 2 of ACT is set, so the plain path pays nothing for it.)
  constexpr bool EXT = (OP == OP_UP || OP == OP_DH) && (ACT & 4) != 0;
  const int nkd = d / WK;
  const int nk = (OP == OP_DW) ? (qe - qb + WK - 1) / WK : ((OP == OP_PART) ? Bs / WK : nkd + (EXT ? 2 : 0));

  // ---- DMA lane roles.  A wavefront issues 4 instructions per operand and stage; instruction
  // (wave, j) fills 1 KiB: for a K-contiguous operand rows 16 (4 wave + j) + lane / 4, physical
  // chunk lane % 4 (logical chunk = physical ^ swizzle(row)); for a K-major operand K-rows
  // 2 (4 wave + j) + lane / 32, physical chunk lane % 32 (logical = physical ^ ((krow & 3) << 2)).
  const uint16_t* a_ptr[4];
  const uint16_t* b_ptr[4];
  int a_coloff[4], b_coloff[4];
  int a_unit[4], b_tok[4];  // K = d GEMMs: hidden unit / token id of this lane's row (for the extension)
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int row = (wave * 4 + j) * 16 + (lane >> 2);
    const int ch = (lane & 3) ^ ((row >> 2) & 3);
    const int krow = 2 * (wave * 4 + j) + (lane >> 5);
    const int kcol = ((lane & 31) ^ ((krow & 3) << 2)) << 3;
    if (!A_TR) {
      const int u = (a0 + row < Bs) ? a0 + row : a0;
      a_ptr[j] = Aop + ((size_t)b * Bs + u) * d + ch * 8;
      a_coloff[j] = 0;
      a_unit[j] = b * Bs + u;
    } else {
      const int col = (a0 + kcol < d) ? a0 + kcol : a0;
      a_coloff[j] = col;
      a_ptr[j] = (OP == OP_PART) ? Aop + ((size_t)b * Bs + krow) * d + col : Aop;
      a_unit[j] = 0;
    }
    if (!B_TR) {
      const int q = (n0 + row < qe) ? n0 + row : n0;
      b_tok[j] = (OP == OP_PART) ? 0 : p.tok[q];
      b_ptr[j] = (OP == OP_PART) ? Bop + (size_t)q * Bs + ch * 8 : Bop + (size_t)b_tok[j] * d + ch * 8;
      b_coloff[j] = 0;
    } else {
      b_coloff[j] = (n0 + kcol < Bs) ? n0 + kcol : n0;
      b_ptr[j] = Bop;
      b_tok[j] = 0;
    }
  }
  const int lane_half = lane >> 5;
  typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;
  const const_i32_ptr tok_c = (const_i32_ptr)(uintptr_t)p.tok;
  // Token ids of the 8 gathered K-rows this wavefront copies per stage (dW only): wave-uniform
  // addresses in the constant address space, so they are scalar loads, which leave the vmcnt
  // bookkeeping of the DMA alone (the ids were written by an earlier launch).  They are
  // fetched one iteration before the copy that needs them is issued.
  auto load_ids = [&](int kt, int (&ids)[8]) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int r0 = qb + kt * WK + 2 * (wave * 4 + j);
      ids[2 * j] = tok_c[min(r0, qe - 1)];
      ids[2 * j + 1] = tok_c[min(r0 + 1, qe - 1)];
    }
  };
  // One DMA instruction: j-th of this wavefront for operand A (which = 0) or B (which = 1),
  // K-stage kt into ring slot `stage`.
  auto issue_one = [&](int which, int j, int stage, int kt, const int (&ids)[8]) {
    const uint32_t dst = __builtin_amdgcn_readfirstlane(
        lds0 + (uint32_t)(stage * W_STAGE + which * W_REGION + (wave * 4 + j) * 1024));
    if (which == 0) {
      if (!A_TR) {
        // (selects, not a branch: the loop body stays one basic block)
        const int ch8 = ((lane & 3) ^ ((lane >> 4) & 3)) * 8;
        const bool ext = EXT && kt >= nkd;
        const uint16_t* src = ext ? p.We + (size_t)a_unit[j] * 64 + (kt - nkd) * WK + ch8 : a_ptr[j] + kt * WK;
        dma16(src, dst);
      } else if (OP == OP_PART) {
        dma16(a_ptr[j] + (size_t)kt * WK * d, dst);
      } else {
        // (arithmetic select: a select between two array elements would be turned into an
        // indexed load from a private-memory copy of the array)
        dma16(Aop + (size_t)(ids[2 * j] + lane_half * (ids[2 * j + 1] - ids[2 * j])) * d + a_coloff[j], dst);
      }
    } else {
      if (!B_TR) {
        const int ch8 = ((lane & 3) ^ ((lane >> 4) & 3)) * 8;
        const bool ext = EXT && kt >= nkd;
        const uint16_t* src = ext ? p.Xe + (size_t)b_tok[j] * 64 + (kt - nkd) * WK + ch8 : b_ptr[j] + kt * WK;
        dma16(src, dst);
      } else {
        const int q = qb + kt * WK + 2 * (wave * 4 + j) + lane_half;
        const uint16_t* src = (q < qe) ? Bop + (size_t)q * Bs + b_coloff[j] : p.zero_row + ((lane & 15) << 3);
        dma16(src, dst);
      }
    }
  };

  // ---- fragment addressing.  Transposing reads, lane (group g = lane / 16, s = lane % 16):
  // K-row 8 (g >> 1) + 4 r + (s >> 2) of the 16-row K-step; column group: natural order
  // 16 (g & 1) + 4 (s & 3) on the B side, the rho32-permuted one on the A side.
  const int g = lane >> 4, sl = lane & 15;
  const int sw = ((sl >> 2) & 3) << 2;
  const int ag = sl & 3;
  const int acol = 4 * (4 * (ag & 1) + 2 * (g & 1) + (ag >> 1));
  const int bcol = 16 * (g & 1) + 4 * (sl & 3);
  const uint32_t tr_row0 = (uint32_t)((8 * (g >> 1) + (sl >> 2)) * 512);
  const int arow = rho32(i);

  // Fragment f of K-step s of the stage at st: f < 4 is A-side tile f, else B-side tile f - 4.
  auto load_frag = [&](const char* st, int s, int f) -> bf16x8 {
    if (f < 4) {
      if (!A_TR) return as_bf16x8(reinterpret_cast<const uint4*>(st)[kd_slot(wm * 128 + f * 32 + arow, 2 * s + h)]);
      const uint32_t ch = (uint32_t)((((wm * 4 + f) * 4 + (acol >> 3)) ^ sw) * 16 + (acol & 4) * 2);
      const char* base = st + s * 16 * 512 + tr_row0 + ch;
      return tr_read_frag(base, base + 4 * 512);
    }
    const char* stB = st + W_REGION;
    if (!B_TR) return as_bf16x8(reinterpret_cast<const uint4*>(stB)[kd_slot(wn * 128 + (f - 4) * 32 + i, 2 * s + h)]);
    const uint32_t ch = (uint32_t)((((wn * 4 + (f - 4)) * 4 + (bcol >> 3)) ^ sw) * 16 + (bcol & 4) * 2);
    const char* base = stB + s * 16 * 512 + tr_row0 + ch;
    return tr_read_frag(base, base + 4 * 512);
  };

  f32x16 acc[4][4];
#pragma unroll
  for (int mi = 0; mi < 4; ++mi)
#pragma unroll
    for (int ni = 0; ni < 4; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;

  // The previous tile's epilogue stores are drained and every wavefront has left its last stage
  // before the ring is refilled.
  wait_vmcnt<0>();
  __builtin_amdgcn_s_barrier();
  // Ring schedule (5 slots).  "Issue j" copies K-stage min(j, nk-1) into slot j % 5: past the
  // last stage it copies the last one again into a slot nobody reads, which keeps the number of
  // copies per iteration -- and with it every vmcnt wait -- the same from the first to the last
  // iteration, and the loop body free of branches.  Issues 0..3 go out up front; iteration kt
  // sends issue kt+4 (into the slot stage kt-1 left).  At the top of iteration kt the stages kt
  // and kt+1 have landed and are visible to every wavefront, and the fragments of (stage kt,
  // K-step 0) are in registers.
  //
  // A wavefront is alone on its SIMD, so nothing hides what it does between two MFMAs: every
  // other instruction of the iteration is therefore placed right behind an MFMA (each keeps the
  // matrix pipe busy for 32 cycles): after MFMA 0..7 of a K-step one fragment read for the next
  // K-step (issued half an iteration before its data are used), after MFMA 8..11 one DMA
  // instruction, after MFMA 12 the scalar loads of the token ids for the next iteration's DMA.
  const int klast = nk - 1;
  auto kclamp = [&](int j) { return j < klast ? j : klast; };
  int ids[8] = {0, 0, 0, 0, 0, 0, 0, 0}, ids_next[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  bf16x8 fa[2][4], fb[2][4];
  const char* ring = reinterpret_cast<const char*>(smem);
  if (nk > 0) {
#pragma unroll
    for (int st = 0; st < 4; ++st) {
      if (OP == OP_DW) load_ids(kclamp(st), ids);
#pragma unroll
      for (int j = 0; j < 4; ++j) issue_one(0, j, st, kclamp(st), ids);
#pragma unroll
      for (int j = 0; j < 4; ++j) issue_one(1, j, st, kclamp(st), ids);
    }
    if (OP == OP_DW) load_ids(kclamp(4), ids);
    wait_vmcnt<16>();  // issues 0 and 1 have landed (2 and 3 may be out)
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int f = 0; f < 4; ++f) {
      fa[0][f] = load_frag(ring, 0, f);
      fb[0][f] = load_frag(ring, 0, f + 4);
    }
  }
  int stage = 0;
  for (int kt = 0; kt < nk; ++kt) {
    const int next = (stage + 1 == W_STAGES) ? 0 : stage + 1;
    const int fill = (stage == 0) ? W_STAGES - 1 : stage - 1;  // slot of stage kt-1 = (kt+4) % 5
    const char* st0 = ring + stage * W_STAGE;
    // after the last stage the look-ahead reads the current one again: harmless
    const char* st1 = ring + ((kt + 1 < nk) ? next : stage) * W_STAGE;
    const int kfill = kclamp(kt + 4);
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      // half 0: multiply K-step 0, read (stage kt, K-step 1), copy the A part of issue kt+4;
      // half 1: multiply K-step 1, read (stage kt+1, K-step 0), copy the B part.
#pragma unroll
      for (int m = 0; m < 16; ++m) {
        const int mi = m >> 2, ni = m & 3;
        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[half][mi], fb[half][ni], acc[mi][ni], 0, 0, 0);
        if (m < 8) {
          const bf16x8 fr = load_frag(half ? st1 : st0, half ? 0 : 1, m);
          if (m < 4) fa[half ^ 1][m] = fr; else fb[half ^ 1][m - 4] = fr;
        } else if (m < 12) {
          issue_one(half, m - 8, fill, kfill, ids);
        } else if (m == 12 && half == 1 && OP == OP_DW) {
          load_ids(kclamp(kt + 5), ids_next);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) ids[e] = ids_next[e];
    // own copies of stage kt+2 have landed: only issues kt+3 and kt+4 (8 instructions each) may
    // be outstanding; the barrier makes everyone's visible and ends all reads of stage kt
    wait_vmcnt<16>();
    __builtin_amdgcn_s_barrier();
    stage = next;
  }
  wait_vmcnt<0>();  // the trailing copies (repeats of the last stage) are done too

  // ---- epilogue: lane (i, h) holds, for B-side index n0 + 128 wn + 32 ni + i, the A-side
  // indices a0 + 128 wm + 32 mi + 16 h + (0..15).
  // dH reads the saved pre-activations of its whole tile first (32 loads of 16 bytes per lane, all
  // in flight together; the fragment registers of the main loop are free by now), so the epilogue
  // waits for memory once instead of once per fragment.
  if (OP == OP_DW) {
    // Stored as they lie, the 64-byte runs of a lane would make an instruction touch 64 lines with
    // 16 bytes each.  Each 32 x 32 tile goes through a wavefront-private LDS buffer (rows of 144
    // bytes; the ring is free once everyone's copies have landed) and comes back with 8 lanes
    // along a row: a store instruction then writes 8 whole 128-byte lines.  (Same wavefront on
    // both sides of the buffer: LDS executes its accesses in order.)
    __builtin_amdgcn_s_barrier();
    float* tbuf = reinterpret_cast<float*>(smem) + wave * (32 * 36);
    const int cc = lane & 7, r0 = lane >> 3;
#pragma unroll
    for (int ni = 0; ni < 4; ++ni)
#pragma unroll
      for (int mi = 0; mi < 4; ++mi) {
        const f32x16& c = acc[mi][ni];
#pragma unroll
        for (int e = 0; e < 4; ++e)
          *reinterpret_cast<f32x4*>(tbuf + i * 36 + 16 * h + 4 * e) = f32x4{c[4 * e], c[4 * e + 1], c[4 * e + 2], c[4 * e + 3]};
        wave_lds_fence();
        const int aidx = a0 + wm * 128 + mi * 32 + 4 * cc;
        f32x4 o[4];  // (all four reads go out before the first store waits for its data)
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = *reinterpret_cast<const f32x4*>(tbuf + (r0 + 8 * e) * 36 + 4 * cc);
        wave_lds_fence();
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int nidx = n0 + wn * 128 + ni * 32 + r0 + 8 * e;
          if (nidx < Bs && aidx < a_lim) *reinterpret_cast<f32x4*>(p.dW + ((size_t)b * Bs + nidx) * d + aidx) = o[e];
        }
      }
    return;
  }
  uint4 zsave[(OP == OP_DH) ? 4 : 1][(OP == OP_DH) ? 4 : 1][2];
  if (OP == OP_DH) {
#pragma unroll
    for (int ni = 0; ni < 4; ++ni) {
      const int nidx = n0 + wn * 128 + ni * 32 + i;
#pragma unroll
      for (int mi = 0; mi < 4; ++mi) {
        const int aidx = a0 + wm * 128 + mi * 32 + 16 * h;
        if (nidx < qe && aidx < a_lim) {
          const uint4* src = reinterpret_cast<const uint4*>(p.Hsave + (size_t)nidx * Bs + aidx);
          zsave[ni][mi][0] = src[0];
          zsave[ni][mi][1] = src[1];
        }
      }
    }
  }
#pragma unroll
  for (int ni = 0; ni < 4; ++ni) {
    const int nidx = n0 + wn * 128 + ni * 32 + i;
    const bool n_ok = (OP == OP_DW) ? nidx < Bs : nidx < qe;
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
      const int aidx = a0 + wm * 128 + mi * 32 + 16 * h;
      const f32x16& c = acc[mi][ni];
      if (n_ok && aidx < a_lim) {
        if (OP == OP_UP) {
          const size_t o = (size_t)nidx * Bs + aidx;
#pragma unroll
          for (int hf = 0; hf < 2; ++hf) {  // 8 values at a time keeps the register need low
            float cv[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) cv[e] = pin_vgpr(c[8 * hf + e]);
            if (!(ACT & 2))  // bit 1 of ACT: inference forward, nothing saved for a backward pass
              reinterpret_cast<uint4*>(p.Hsave + o)[hf] =
                  make_uint4(pack_bf16x2(cv[0], cv[1]), pack_bf16x2(cv[2], cv[3]),
                             pack_bf16x2(cv[4], cv[5]), pack_bf16x2(cv[6], cv[7]));
            reinterpret_cast<uint4*>(p.Hact + o)[hf] =
                make_uint4(pack_bf16x2(act_fn<(ACT & 1)>(cv[0]), act_fn<(ACT & 1)>(cv[1])),
                           pack_bf16x2(act_fn<(ACT & 1)>(cv[2]), act_fn<(ACT & 1)>(cv[3])),
                           pack_bf16x2(act_fn<(ACT & 1)>(cv[4]), act_fn<(ACT & 1)>(cv[5])),
                           pack_bf16x2(act_fn<(ACT & 1)>(cv[6]), act_fn<(ACT & 1)>(cv[7])));
            __builtin_amdgcn_sched_barrier(0);
          }
        } else if (OP == OP_DH) {
          const size_t o = (size_t)nidx * Bs + aidx;
#pragma unroll
          for (int hf = 0; hf < 2; ++hf) {
            float cv[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) cv[e] = pin_vgpr(c[8 * hf + e]);
            const uint4 z = zsave[(OP == OP_DH) ? ni : 0][(OP == OP_DH) ? mi : 0][hf];
            const uint32_t zw[4] = {z.x, z.y, z.z, z.w};
            uint32_t gv[4], av[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float zl = lo_bf16(zw[e]), zh = hi_bf16(zw[e]);
              gv[e] = pack_bf16x2(cv[2 * e] * act_grad<(ACT & 1)>(zl), cv[2 * e + 1] * act_grad<(ACT & 1)>(zh));
              av[e] = pack_bf16x2(act_fn<(ACT & 1)>(zl), act_fn<(ACT & 1)>(zh));
            }
            reinterpret_cast<uint4*>(p.dHpre + o)[hf] = make_uint4(gv[0], gv[1], gv[2], gv[3]);
            reinterpret_cast<uint4*>(p.Hact + o)[hf] = make_uint4(av[0], av[1], av[2], av[3]);
            __builtin_amdgcn_sched_barrier(0);
          }
        } else if (OP == OP_PART) {
          uint4* dst = reinterpret_cast<uint4*>(p.part + (size_t)nidx * d + aidx);
          dst[0] = make_uint4(pack_bf16x2(c[0], c[1]), pack_bf16x2(c[2], c[3]), pack_bf16x2(c[4], c[5]),
                              pack_bf16x2(c[6], c[7]));
          dst[1] = make_uint4(pack_bf16x2(c[8], c[9]), pack_bf16x2(c[10], c[11]),
                              pack_bf16x2(c[12], c[13]), pack_bf16x2(c[14], c[15]));
        }
      }
    }
  }
}

// Up / dH / partial-row GEMMs: persistent workgroups, one per CU.  Workgroup id modulo 8 is
// the XCD it runs on; it walks that XCD's work items -- (row tile of the XCD's list, A-side
// tile), in groups of W_RT row tiles x all A-side tiles, A-side tile major -- with a stride of
// the workgroups per XCD.  The 32 workgroups of an XCD are then on about 4 row tiles x 8
// A-side tiles at a time, in step, so each operand slice pulled into that XCD's L2 serves
// several of them.
template <int OP, int ACT>
__global__ __launch_bounds__(256, 1) void wide_rows_kernel(WideArgs p) {
  extern __shared__ uint4 w_smem[];
  const int xcd = blockIdx.x & 7, wg_per_xcd = gridDim.x >> 3;
  const int count = p.kd_count[xcd];
  const int a_lim = (OP == OP_PART) ? p.d : p.Bs;
  const int n_at = (a_lim + WD - 1) / WD;
  const KdTile* list = static_cast<const KdTile*>(p.kd_list) + (size_t)xcd * p.cap;
  for (int item = blockIdx.x >> 3; item < count * n_at; item += wg_per_xcd) {
    const int grp = item / (W_RT * n_at), rem = item - grp * W_RT * n_at;
    const int rtg = (count - grp * W_RT < W_RT) ? count - grp * W_RT : W_RT;
    const KdTile t = list[grp * W_RT + rem % rtg];
    wide_tile<OP, ACT>(p, w_smem, t.bucket, (rem / rtg) * WD, t.q0, 0, p.offsets[t.bucket + 1]);
  }
}

// dW GEMMs: one work item (column tile, unit tile, bucket) per workgroup.  With a multiple of
// 8 column tiles an XCD keeps to the column tiles congruent to its id and takes, for each
// bucket (largest first), all unit tiles of one column tile side by side: they gather the same
// 512-byte column slab of the same activation rows.
__global__ __launch_bounds__(256, 1) void wide_dw_kernel(WideArgs p) {
  extern __shared__ uint4 w_smem[];
  const int n_ct = (p.d + WD - 1) / WD, n_ut = (p.Bs + WD - 1) / WD;
  int ct, ut, br;
  if (n_ct % 8 == 0) {
    const int xcd = blockIdx.x & 7, jj = blockIdx.x >> 3, per = n_ct / 8;
    ut = jj % n_ut;
    const int r = jj / n_ut;
    ct = xcd + 8 * (r % per);
    br = r / per;
  } else {
    ut = blockIdx.x % n_ut;
    const int r = blockIdx.x / n_ut;
    ct = r % n_ct;
    br = r / n_ct;
  }
  if (br >= p.N) return;
  const int b = p.border[br];
  wide_tile<OP_DW, 0>(p, w_smem, b, ct * WD, ut * WD, p.offsets[b], p.offsets[b + 1]);
}

template <int OP, int ACT>
static void launch_rows(const WideArgs& a, hipStream_t st) {
  (void)hipFuncSetAttribute(reinterpret_cast<const void*>(wide_rows_kernel<OP, ACT>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, W_SMEM);
  wide_rows_kernel<OP, ACT><<<8 * 32, 256, W_SMEM, st>>>(a);
}

hipError_t launch_wide(int op, const spt_shape_t& s, const WideArgs& a, hipStream_t st) {
  const bool gelu = s.act == SPT_ACT_GELU;
  switch (op) {
    case OP_UP:  // the activation code's bit 1 marks the inference forward (no Hsave), bit 2
                 // the low-rank extension of the K loop
      if (a.Xe)         { if (gelu) launch_rows<OP_UP, 4>(a, st); else launch_rows<OP_UP, 5>(a, st); }
      else if (a.Hsave) { if (gelu) launch_rows<OP_UP, 0>(a, st); else launch_rows<OP_UP, 1>(a, st); }
      else              { if (gelu) launch_rows<OP_UP, 2>(a, st); else launch_rows<OP_UP, 3>(a, st); }
      break;
    case OP_DH:
      if (a.Xe) { if (gelu) launch_rows<OP_DH, 4>(a, st); else launch_rows<OP_DH, 5>(a, st); }
      else      { if (gelu) launch_rows<OP_DH, 0>(a, st); else launch_rows<OP_DH, 1>(a, st); }
      break;
    case OP_PART:
      launch_rows<OP_PART, 0>(a, st);
      break;
    default: {
      const int n_ct = (s.d + WD - 1) / WD, n_ut = (s.Bs + WD - 1) / WD;
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(wide_dw_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, W_SMEM);
      wide_dw_kernel<<<n_ct * n_ut * s.N, 256, W_SMEM, st>>>(a);
    }
  }
  return hipGetLastError();
}

}  // namespace spt
