// Grouped bf16 MFMA GEMMs of the routed FFN and the deterministic combine.
//
// Algorithm 4 of the paper runs, per weight block, a gather, two dense GEMMs and a scatter.
// Here every stage is ONE launch over all blocks: a row tile knows its bucket from a small
// prefix table built on the device, the gather is fused into the operand loads, and block
// outputs are written as per-pair partial rows that a fixed-order sum folds into Y (or dX).
//
// All five GEMM stages share one core: a 128x128 output tile per workgroup (4 wavefronts,
// 64x64 each, v_mfma_f32_32x32x16_bf16), both operands staged in LDS as [row][64 K-values]
// with K contiguous, so fragments are plain 16-byte LDS reads.  Operands that arrive with K
// as the strided dimension (weights in the down/dX GEMMs, everything in the dW GEMMs) are
// transposed in registers, 8x8 values per lane, on their way into LDS.
//
// The MFMA "row" dimension is always the one that is contiguous in the output tensor, so a
// lane's four consecutive accumulator rows become one vector store.
#include "spt_device.hpp"
#include "spt_host.hpp"
#include "profile.hpp"

namespace spt {

constexpr int KT = 64;     // K values per LDS tile row
constexpr int TILE = 128;  // output tile edge

// 16-byte slot of (row, chunk) in an LDS tile of 8 chunks per row.  The XOR spreads both the
// fragment reads (32 consecutive rows, same chunk) and the transposed writes (rows 8 apart,
// same chunk) over the banks.
__device__ __forceinline__ int lds_slot(int row, int chunk) {
  return row * 8 + (chunk ^ (((row >> 1) & 7) ^ ((row >> 4) & 3)));
}

__device__ __forceinline__ bf16x8 as_bf16x8(const uint4& v) { return __builtin_bit_cast(bf16x8, v); }

// acc[mi][ni] += A[arow0 + 32 mi .. , :] * B[brow0 + 32 ni .. , :]^T over one 64-wide K tile.
template <int MI, int NI>
__device__ __forceinline__ void mma_ktile(const uint4* As, const uint4* Bs, int arow0, int brow0,
                                          int lane, f32x16 (&acc)[MI][NI]) {
  const int i = lane & 31, h = lane >> 5;
#pragma unroll
  for (int s = 0; s < KT / 16; ++s) {
    bf16x8 a[MI], b[NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) a[mi] = as_bf16x8(As[lds_slot(arow0 + mi * 32 + i, 2 * s + h)]);
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) b[ni] = as_bf16x8(Bs[lds_slot(brow0 + ni * 32 + i, 2 * s + h)]);
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mi], b[ni], acc[mi][ni], 0, 0, 0);
  }
}

// in[kk] holds 8 consecutive n-values of K-row kk; out[r] gets the 8 K-values of n-row r.
__device__ __forceinline__ void transpose8x8(const uint4 (&in)[8], uint4 (&out)[8]) {
  const uint32_t* s = reinterpret_cast<const uint32_t*>(in);  // s[kk*4 + c]: n = 2c (lo), 2c+1 (hi)
  uint32_t* o = reinterpret_cast<uint32_t*>(out);             // o[r*4 + c']: k = 2c' (lo), 2c'+1 (hi)
#pragma unroll
  for (int c = 0; c < 4; ++c)
#pragma unroll
    for (int cp = 0; cp < 4; ++cp) {
      const uint32_t even = s[(2 * cp) * 4 + c], odd = s[(2 * cp + 1) * 4 + c];
      o[(2 * c) * 4 + cp] = (even & 0xFFFFu) | (odd << 16);          // low halves
      o[(2 * c + 1) * 4 + cp] = (even >> 16) | (odd & 0xFFFF0000u);  // high halves
    }
}

__device__ __forceinline__ uint4 ldg16(const uint16_t* p) {
  return p ? *reinterpret_cast<const uint4*>(p) : make_uint4(0u, 0u, 0u, 0u);
}

// Which bucket owns row tile `tile`: the largest b with tile_prefix[b] <= tile.
__device__ __forceinline__ int find_bucket(const int32_t* __restrict__ tile_prefix, int N, int tile) {
  int lo = 0, hi = N;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (tile_prefix[mid] <= tile) lo = mid; else hi = mid;
  }
  return lo;
}

// ------------------------------------------------------------------------------------------
// tile table and token ids
__global__ __launch_bounds__(1024) void plan_kernel(const int32_t* __restrict__ offsets, int N,
                                                    int32_t* __restrict__ tile_prefix) {
  __shared__ int32_t scan[1024];
  const int b = threadIdx.x;
  const int nt = (b < N) ? (offsets[b + 1] - offsets[b] + kRowTile - 1) / kRowTile : 0;
  scan[b] = nt;
  __syncthreads();
  for (int s = 1; s < 1024; s <<= 1) {
    const int v = (b >= s) ? scan[b - s] : 0;
    __syncthreads();
    scan[b] += v;
    __syncthreads();
  }
  if (b < N) tile_prefix[b] = scan[b] - nt;
  if (b == N - 1) tile_prefix[N] = scan[b];
}

__global__ void tok_kernel(const int32_t* __restrict__ perm, int P, int k, int32_t* __restrict__ tok) {
  const int q = blockIdx.x * blockDim.x + threadIdx.x;
  if (q < P) tok[q] = perm[q] / k;
}

// ------------------------------------------------------------------------------------------
// K = d GEMMs: up-projection (MODE 0) and dH (MODE 1).
//   C[u][q] = sum_i W[b][u][i] * Act[tok[q]][i]      rows u = hidden unit, cols q = bucket row
// MODE 0 (Alg. 4 inner projection): Hsave <- C (if given), Hact <- act(C).
// MODE 1 (backward):                dHpre <- C * act'(Hsave), Hact <- act(Hsave).
template <int MODE, int ACT>
__global__ __launch_bounds__(256) void kd_gemm_kernel(
    const uint16_t* __restrict__ W, const uint16_t* __restrict__ Act,
    const int32_t* __restrict__ offsets, const int32_t* __restrict__ tile_prefix,
    const int32_t* __restrict__ tok, int N, int Bs, int d, uint16_t* __restrict__ Hsave,
    uint16_t* __restrict__ Hact, uint16_t* __restrict__ dHpre) {
  __shared__ uint4 As[TILE * 8];
  __shared__ uint4 Bt[TILE * 8];
  const int tile = blockIdx.x;
  if (tile >= tile_prefix[N]) return;
  const int b = find_bucket(tile_prefix, N, tile);
  const int q0 = offsets[b] + (tile - tile_prefix[b]) * kRowTile;
  const int qend = offsets[b + 1];
  const int u0 = blockIdx.y * TILE;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  const uint16_t* aptr[4];
  const uint16_t* bptr[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = (tid >> 3) + 32 * i;
    const int u = u0 + row, q = q0 + row;
    aptr[i] = (u < Bs) ? W + ((size_t)b * Bs + u) * d + (tid & 7) * 8 : nullptr;
    bptr[i] = (q < qend) ? Act + (size_t)tok[q] * d + (tid & 7) * 8 : nullptr;
  }
  f32x16 acc[2][2];
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;

  uint4 ra[4], rb[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    ra[i] = ldg16(aptr[i]);
    rb[i] = ldg16(bptr[i]);
  }
  for (int k0 = 0; k0 < d; k0 += KT) {
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = (tid >> 3) + 32 * i;
      As[lds_slot(row, tid & 7)] = ra[i];
      Bt[lds_slot(row, tid & 7)] = rb[i];
    }
    __syncthreads();
    if (k0 + KT < d) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        ra[i] = ldg16(aptr[i] ? aptr[i] + k0 + KT : nullptr);
        rb[i] = ldg16(bptr[i] ? bptr[i] + k0 + KT : nullptr);
      }
    }
    mma_ktile<2, 2>(As, Bt, wm * 64, wn * 64, lane, acc);
  }

  const int i = lane & 31, h = lane >> 5;
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) {
      const int q = q0 + wn * 64 + ni * 32 + i;
      if (q >= qend) continue;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int u = u0 + wm * 64 + mi * 32 + 8 * g + 4 * h;
        if (u >= Bs) continue;
        const size_t o = (size_t)q * Bs + u;
        const float c0 = acc[mi][ni][4 * g], c1 = acc[mi][ni][4 * g + 1];
        const float c2 = acc[mi][ni][4 * g + 2], c3 = acc[mi][ni][4 * g + 3];
        if (MODE == 0) {
          if (Hsave) *reinterpret_cast<uint2*>(Hsave + o) = make_uint2(pack_bf16x2(c0, c1), pack_bf16x2(c2, c3));
          *reinterpret_cast<uint2*>(Hact + o) =
              make_uint2(pack_bf16x2(act_fn<ACT>(c0), act_fn<ACT>(c1)),
                         pack_bf16x2(act_fn<ACT>(c2), act_fn<ACT>(c3)));
        } else {
          const uint2 hp = *reinterpret_cast<const uint2*>(Hsave + o);
          const float z0 = lo_bf16(hp.x), z1 = hi_bf16(hp.x), z2 = lo_bf16(hp.y), z3 = hi_bf16(hp.y);
          *reinterpret_cast<uint2*>(dHpre + o) =
              make_uint2(pack_bf16x2(c0 * act_grad<ACT>(z0), c1 * act_grad<ACT>(z1)),
                         pack_bf16x2(c2 * act_grad<ACT>(z2), c3 * act_grad<ACT>(z3)));
          *reinterpret_cast<uint2*>(Hact + o) =
              make_uint2(pack_bf16x2(act_fn<ACT>(z0), act_fn<ACT>(z1)),
                         pack_bf16x2(act_fn<ACT>(z2), act_fn<ACT>(z3)));
        }
      }
    }
}

// ------------------------------------------------------------------------------------------
// K = Bs GEMMs: down-projection (Alg. 4 outer projection, W = W2, Hin = act(H)) and the dX
// partials (W = W1, Hin = dHpre).
//   part[q][c] = sum_u Hin[q][u] * W[b][u][c]      rows c = output column, cols q = bucket row
__global__ __launch_bounds__(256) void kb_gemm_kernel(
    const uint16_t* __restrict__ W, const uint16_t* __restrict__ Hin,
    const int32_t* __restrict__ offsets, const int32_t* __restrict__ tile_prefix, int N, int Bs,
    int d, uint16_t* __restrict__ part) {
  __shared__ uint4 As[TILE * 8];
  __shared__ uint4 Bt[TILE * 8];
  const int tile = blockIdx.x;
  if (tile >= tile_prefix[N]) return;
  const int b = find_bucket(tile_prefix, N, tile);
  const int q0 = offsets[b] + (tile - tile_prefix[b]) * kRowTile;
  const int qend = offsets[b + 1];
  const int c0 = blockIdx.y * TILE;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  // A: transposing loader, threads 0..127, an 8(k) x 8(c) patch each.
  const int nb = tid & 15, kb = (tid >> 4) & 7;
  const bool a_thread = tid < 128 && (c0 + 8 * nb) < d;
  const uint16_t* abase = W + (size_t)b * Bs * d + c0 + 8 * nb;
  // B: straight copy of Hin rows.
  const uint16_t* bptr[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int q = q0 + (tid >> 3) + 32 * i;
    bptr[i] = (q < qend) ? Hin + (size_t)q * Bs + (tid & 7) * 8 : nullptr;
  }
  f32x16 acc[2][2];
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;

  for (int k0 = 0; k0 < Bs; k0 += KT) {
    uint4 in[8], out[8], rb[4];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      const int u = k0 + 8 * kb + kk;
      in[kk] = ldg16((a_thread && u < Bs) ? abase + (size_t)u * d : nullptr);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
      rb[i] = ldg16((bptr[i] && (k0 + (tid & 7) * 8) < Bs) ? bptr[i] + k0 : nullptr);
    transpose8x8(in, out);
    __syncthreads();
    if (tid < 128) {
#pragma unroll
      for (int r = 0; r < 8; ++r) As[lds_slot(8 * nb + r, kb)] = out[r];
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) Bt[lds_slot((tid >> 3) + 32 * i, tid & 7)] = rb[i];
    __syncthreads();
    mma_ktile<2, 2>(As, Bt, wm * 64, wn * 64, lane, acc);
  }

  const int i = lane & 31, h = lane >> 5;
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) {
      const int q = q0 + wn * 64 + ni * 32 + i;
      if (q >= qend) continue;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int c = c0 + wm * 64 + mi * 32 + 8 * g + 4 * h;
        if (c >= d) continue;
        *reinterpret_cast<uint2*>(part + (size_t)q * d + c) =
            make_uint2(pack_bf16x2(acc[mi][ni][4 * g], acc[mi][ni][4 * g + 1]),
                       pack_bf16x2(acc[mi][ni][4 * g + 2], acc[mi][ni][4 * g + 3]));
      }
    }
}

// ------------------------------------------------------------------------------------------
// K = Bs GEMMs for Bs <= 128, the output-write-bound shape of the benchmark workloads.
// One workgroup owns 128 bucket rows and walks over ALL output columns in chunks of 128:
// the Hin tile (128 rows x Bs) is read once and stays in LDS, each weight chunk (Bs x 128
// columns) is transposed on its way into LDS, and every finished 128x128 chunk is staged
// through LDS so that 16 lanes write 256 contiguous bytes of one partial row.
// MFMA row i of a 32-row tile is fed weight column rho(i) = 16*((i>>2)&1) + 4*(i>>3) + (i&3),
// which makes the 16 accumulator values of a lane 16 CONSECUTIVE output columns.
__device__ __forceinline__ int rho32(int i) { return 16 * ((i >> 2) & 1) + 4 * (i >> 3) + (i & 3); }

__global__ __launch_bounds__(256, 2) void kb_gemm_rows_kernel(
    const uint16_t* __restrict__ W, const uint16_t* __restrict__ Hin,
    const int32_t* __restrict__ offsets, const int32_t* __restrict__ tile_prefix, int N, int Bs,
    int d, uint16_t* __restrict__ part) {
  __shared__ uint4 Ht[2 * TILE * 8];  // [K half][row q][8 chunks]
  __shared__ uint4 As[2 * TILE * 8];  // [K half][row c][8 chunks]; then [row q][16 slots] staging
  const int tile = blockIdx.x;
  if (tile >= tile_prefix[N]) return;
  const int b = find_bucket(tile_prefix, N, tile);
  const int q0 = offsets[b] + (tile - tile_prefix[b]) * kRowTile;
  const int qend = offsets[b + 1];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int i = lane & 31, h = lane >> 5;

#pragma unroll
  for (int it = 0; it < 8; ++it) {
    const int sid = tid + 256 * it;
    const int row = sid >> 4, ch = sid & 15;
    const int q = q0 + row;
    const bool ok = q < qend && ch * 8 < Bs;
    Ht[(ch >> 3) * TILE * 8 + lds_slot(row, ch & 7)] = ldg16(ok ? Hin + (size_t)q * Bs + ch * 8 : nullptr);
  }
  const int nb = tid & 15, kb = tid >> 4;  // this thread's 8(k) x 8(c) weight patch
  const uint16_t* wbase = W + (size_t)b * Bs * d + (size_t)(8 * kb) * d + 8 * nb;
  const bool k_ok = 8 * kb < Bs;
  const int ksteps = Bs / 16;
  const int nchunks = (d + TILE - 1) / TILE;

  uint4 in[8], out[8];
#pragma unroll
  for (int kk = 0; kk < 8; ++kk)
    in[kk] = ldg16((k_ok && 8 * nb < d) ? wbase + (size_t)kk * d : nullptr);

  for (int cc = 0; cc < nchunks; ++cc) {
    const int c0 = cc * TILE;
    transpose8x8(in, out);
    __syncthreads();  // staging reads of the previous chunk are done
#pragma unroll
    for (int r = 0; r < 8; ++r) As[(kb >> 3) * TILE * 8 + lds_slot(8 * nb + r, kb & 7)] = out[r];
    __syncthreads();
    if (cc + 1 < nchunks) {
      const bool ok = k_ok && (c0 + TILE + 8 * nb) < d;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) in[kk] = ldg16(ok ? wbase + (size_t)kk * d + c0 + TILE : nullptr);
    }
    f32x16 acc[2][2];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
      for (int ni = 0; ni < 2; ++ni)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;
    for (int s = 0; s < ksteps; ++s) {
      const int half = (s >> 2) * TILE * 8, ch = 2 * (s & 3) + h;
      bf16x8 a[2], bb[2];
#pragma unroll
      for (int mi = 0; mi < 2; ++mi) a[mi] = as_bf16x8(As[half + lds_slot(wm * 64 + mi * 32 + rho32(i), ch)]);
#pragma unroll
      for (int ni = 0; ni < 2; ++ni) bb[ni] = as_bf16x8(Ht[half + lds_slot(wn * 64 + ni * 32 + i, ch)]);
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mi], bb[ni], acc[mi][ni], 0, 0, 0);
    }
    __syncthreads();  // every wavefront is done reading As
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
      for (int ni = 0; ni < 2; ++ni) {
        const int q = wn * 64 + ni * 32 + i;
        const int slot = (wm * 64 + mi * 32 + 16 * h) >> 3;
        const f32x16& c = acc[mi][ni];
        As[q * 16 + (slot ^ (q & 15))] =
            make_uint4(pack_bf16x2(c[0], c[1]), pack_bf16x2(c[2], c[3]), pack_bf16x2(c[4], c[5]),
                       pack_bf16x2(c[6], c[7]));
        As[q * 16 + ((slot + 1) ^ (q & 15))] =
            make_uint4(pack_bf16x2(c[8], c[9]), pack_bf16x2(c[10], c[11]),
                       pack_bf16x2(c[12], c[13]), pack_bf16x2(c[14], c[15]));
      }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int sid = tid + 256 * it;
      const int q = sid >> 4, slot = sid & 15;
      if (q0 + q < qend && c0 + 8 * slot < d)
        *reinterpret_cast<uint4*>(part + (size_t)(q0 + q) * d + c0 + 8 * slot) = As[q * 16 + (slot ^ (q & 15))];
    }
  }
}

// ------------------------------------------------------------------------------------------
// K = bucket rows GEMMs: dW1 (Act = X, Hin = dHpre) and dW2 (Act = dY, Hin = act(H)).
//   dW[b][u][c] = sum_{q in bucket b} Hin[q][u] * Act[tok[q]][c]    rows c, cols u
// K runs over the bucket's rows in sorted order, so the sum order is fixed.
__global__ __launch_bounds__(256) void kq_gemm_kernel(
    const uint16_t* __restrict__ Act, const uint16_t* __restrict__ Hin,
    const int32_t* __restrict__ offsets, const int32_t* __restrict__ tok, int Bs, int d,
    float* __restrict__ dW) {
  __shared__ uint4 As[TILE * 8];
  __shared__ uint4 Bt[TILE * 8];
  const int b = blockIdx.y;
  const int c0 = blockIdx.x * TILE, u0 = blockIdx.z * TILE;
  const int qb = offsets[b], qe = offsets[b + 1];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int t2 = tid & 127;
  const int nb = t2 & 15, kb = t2 >> 4;
  const bool is_a = tid < 128;
  const bool col_ok = is_a ? (c0 + 8 * nb) < d : (u0 + 8 * nb) < Bs;

  f32x16 acc[2][2];
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;

  for (int k0 = qb; k0 < qe; k0 += KT) {
    uint4 in[8], out[8];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      const int q = k0 + 8 * kb + kk;
      const uint16_t* p = nullptr;
      if (col_ok && q < qe)
        p = is_a ? Act + (size_t)tok[q] * d + c0 + 8 * nb : Hin + (size_t)q * Bs + u0 + 8 * nb;
      in[kk] = ldg16(p);
    }
    transpose8x8(in, out);
    __syncthreads();
    uint4* dst = is_a ? As : Bt;
#pragma unroll
    for (int r = 0; r < 8; ++r) dst[lds_slot(8 * nb + r, kb)] = out[r];
    __syncthreads();
    mma_ktile<2, 2>(As, Bt, wm * 64, wn * 64, lane, acc);
  }

  const int i = lane & 31, h = lane >> 5;
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) {
      const int u = u0 + wn * 64 + ni * 32 + i;
      if (u >= Bs) continue;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int c = c0 + wm * 64 + mi * 32 + 8 * g + 4 * h;
        if (c >= d) continue;
        f32x4 v = {acc[mi][ni][4 * g], acc[mi][ni][4 * g + 1], acc[mi][ni][4 * g + 2],
                   acc[mi][ni][4 * g + 3]};
        *reinterpret_cast<f32x4*>(dW + ((size_t)b * Bs + u) * d + c) = v;
      }
    }
}

// ------------------------------------------------------------------------------------------
// Combine: out[t][:] = sum_{j<k} part[inv[t*k+j]][:], j ascending, fp32, one rounding to bf16.
// This is Alg. 4's write-back with block outputs added (k > 1 blocks per token).
__global__ __launch_bounds__(256) void combine_kernel(const uint16_t* __restrict__ part,
                                                      const int32_t* __restrict__ inv, int T, int d,
                                                      int k, uint16_t* __restrict__ out) {
  const int cpr = d >> 3;  // 16-byte groups per row
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= (int64_t)T * cpr) return;
  const int t = (int)(gid / cpr), cg = (int)(gid % cpr);
  float a[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) a[e] = 0.f;
  const int32_t* iv = inv + (size_t)t * k;
  int j = 0;
  for (; j + 4 <= k; j += 4) {
    uint4 v[4];
#pragma unroll
    for (int jj = 0; jj < 4; ++jj)
      v[jj] = *reinterpret_cast<const uint4*>(part + (size_t)iv[j + jj] * d + cg * 8);
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      a[0] += lo_bf16(v[jj].x); a[1] += hi_bf16(v[jj].x);
      a[2] += lo_bf16(v[jj].y); a[3] += hi_bf16(v[jj].y);
      a[4] += lo_bf16(v[jj].z); a[5] += hi_bf16(v[jj].z);
      a[6] += lo_bf16(v[jj].w); a[7] += hi_bf16(v[jj].w);
    }
  }
  for (; j < k; ++j) {
    const uint4 v = *reinterpret_cast<const uint4*>(part + (size_t)iv[j] * d + cg * 8);
    a[0] += lo_bf16(v.x); a[1] += hi_bf16(v.x);
    a[2] += lo_bf16(v.y); a[3] += hi_bf16(v.y);
    a[4] += lo_bf16(v.z); a[5] += hi_bf16(v.z);
    a[6] += lo_bf16(v.w); a[7] += hi_bf16(v.w);
  }
  *reinterpret_cast<uint4*>(out + (size_t)t * d + cg * 8) =
      make_uint4(pack_bf16x2(a[0], a[1]), pack_bf16x2(a[2], a[3]), pack_bf16x2(a[4], a[5]),
                 pack_bf16x2(a[6], a[7]));
}

// ------------------------------------------------------------------------------------------
// host side
static int max_row_tiles(const spt_shape_t& s) {
  const int64_t P = (int64_t)s.T * s.k;
  return (int)((P + kRowTile - 1) / kRowTile) + s.N;
}

FwdWorkspace plan_fwd(const spt_shape_t& s, void* ws) {
  const size_t P = (size_t)s.T * s.k;
  char* p = static_cast<char*>(ws);
  size_t o = 0;
  FwdWorkspace w;
  w.tile_prefix = reinterpret_cast<int32_t*>(p + o); o += align256((size_t)(s.N + 1) * 4);
  w.tok = reinterpret_cast<int32_t*>(p + o);         o += align256(P * 4);
  w.Hact = reinterpret_cast<uint16_t*>(p + o);       o += align256(P * s.Bs * 2);
  w.part = reinterpret_cast<uint16_t*>(p + o);       o += align256(P * s.d * 2);
  w.bytes = o;
  return w;
}

BwdWorkspace plan_bwd(const spt_shape_t& s, void* ws) {
  const size_t P = (size_t)s.T * s.k;
  char* p = static_cast<char*>(ws);
  size_t o = 0;
  BwdWorkspace w;
  w.tile_prefix = reinterpret_cast<int32_t*>(p + o); o += align256((size_t)(s.N + 1) * 4);
  w.tok = reinterpret_cast<int32_t*>(p + o);         o += align256(P * 4);
  w.Hact = reinterpret_cast<uint16_t*>(p + o);       o += align256(P * s.Bs * 2);
  w.dHpre = reinterpret_cast<uint16_t*>(p + o);      o += align256(P * s.Bs * 2);
  w.part = reinterpret_cast<uint16_t*>(p + o);       o += align256(P * s.d * 2);
  w.bytes = o;
  return w;
}

#define SPT_LAUNCH_CHECK()                 \
  do {                                     \
    hipError_t e_ = hipGetLastError();     \
    if (e_ != hipSuccess) return e_;       \
  } while (0)

static hipError_t run_plan(const spt_shape_t& s, const int32_t* offsets, const int32_t* perm,
                           int32_t* tile_prefix, int32_t* tok, hipStream_t st) {
  const int P = s.T * s.k;
  {
    ScopedKernelTimer tm(kSlotPlan, st);
    plan_kernel<<<1, 1024, 0, st>>>(offsets, s.N, tile_prefix);
  }
  SPT_LAUNCH_CHECK();
  {
    ScopedKernelTimer tm(kSlotTok, st);
    tok_kernel<<<(P + 255) / 256, 256, 0, st>>>(perm, P, s.k, tok);
  }
  SPT_LAUNCH_CHECK();
  return hipSuccess;
}

static hipError_t run_combine(const spt_shape_t& s, const uint16_t* part, const int32_t* inv,
                              void* out, int slot, hipStream_t st) {
  const int64_t items = (int64_t)s.T * (s.d / 8);
  ScopedKernelTimer tm(slot, st);
  combine_kernel<<<(unsigned)((items + 255) / 256), 256, 0, st>>>(part, inv, s.T, s.d, s.k,
                                                                  static_cast<uint16_t*>(out));
  SPT_LAUNCH_CHECK();
  return hipSuccess;
}

hipError_t run_fwd(const spt_shape_t& s, const void* X, const void* W1, const void* W2,
                   const int32_t* offsets, const int32_t* perm, const int32_t* inv, void* Y,
                   void* Hsave, const FwdWorkspace& w, hipStream_t st) {
  hipError_t e = run_plan(s, offsets, perm, w.tile_prefix, w.tok, st);
  if (e != hipSuccess) return e;
  const int tiles = max_row_tiles(s);
  const dim3 g1(tiles, (s.Bs + TILE - 1) / TILE);
  auto x = static_cast<const uint16_t*>(X);
  auto w1 = static_cast<const uint16_t*>(W1);
  auto w2 = static_cast<const uint16_t*>(W2);
  auto hs = static_cast<uint16_t*>(Hsave);
  {
    ScopedKernelTimer tm(kSlotUp, st);
    if (s.act == SPT_ACT_GELU)
      kd_gemm_kernel<0, 0><<<g1, 256, 0, st>>>(w1, x, offsets, w.tile_prefix, w.tok, s.N, s.Bs,
                                               s.d, hs, w.Hact, nullptr);
    else
      kd_gemm_kernel<0, 1><<<g1, 256, 0, st>>>(w1, x, offsets, w.tile_prefix, w.tok, s.N, s.Bs,
                                               s.d, hs, w.Hact, nullptr);
  }
  SPT_LAUNCH_CHECK();
  const dim3 g2(tiles, (s.d + TILE - 1) / TILE);
  {
    ScopedKernelTimer tm(kSlotDown, st);
    if (s.Bs <= TILE)
      kb_gemm_rows_kernel<<<tiles, 256, 0, st>>>(w2, w.Hact, offsets, w.tile_prefix, s.N, s.Bs, s.d, w.part);
    else
      kb_gemm_kernel<<<g2, 256, 0, st>>>(w2, w.Hact, offsets, w.tile_prefix, s.N, s.Bs, s.d, w.part);
  }
  SPT_LAUNCH_CHECK();
  return run_combine(s, w.part, inv, Y, kSlotCombineY, st);
}

hipError_t run_bwd(const spt_shape_t& s, const void* X, const void* W1, const void* W2,
                   const void* dY, const int32_t* offsets, const int32_t* perm,
                   const int32_t* inv, const void* Hsave, void* dX, float* dW1, float* dW2,
                   const BwdWorkspace& w, hipStream_t st) {
  hipError_t e = run_plan(s, offsets, perm, w.tile_prefix, w.tok, st);
  if (e != hipSuccess) return e;
  const int tiles = max_row_tiles(s);
  auto x = static_cast<const uint16_t*>(X);
  auto w1 = static_cast<const uint16_t*>(W1);
  auto w2 = static_cast<const uint16_t*>(W2);
  auto dy = static_cast<const uint16_t*>(dY);
  auto hs = const_cast<uint16_t*>(static_cast<const uint16_t*>(Hsave));
  const dim3 g1(tiles, (s.Bs + TILE - 1) / TILE);
  {
    ScopedKernelTimer tm(kSlotDH, st);
    if (s.act == SPT_ACT_GELU)
      kd_gemm_kernel<1, 0><<<g1, 256, 0, st>>>(w2, dy, offsets, w.tile_prefix, w.tok, s.N, s.Bs,
                                               s.d, hs, w.Hact, w.dHpre);
    else
      kd_gemm_kernel<1, 1><<<g1, 256, 0, st>>>(w2, dy, offsets, w.tile_prefix, w.tok, s.N, s.Bs,
                                               s.d, hs, w.Hact, w.dHpre);
  }
  SPT_LAUNCH_CHECK();
  const dim3 g3((s.d + TILE - 1) / TILE, s.N, (s.Bs + TILE - 1) / TILE);
  {
    ScopedKernelTimer tm(kSlotDW2, st);
    kq_gemm_kernel<<<g3, 256, 0, st>>>(dy, w.Hact, offsets, w.tok, s.Bs, s.d, dW2);
  }
  SPT_LAUNCH_CHECK();
  {
    ScopedKernelTimer tm(kSlotDW1, st);
    kq_gemm_kernel<<<g3, 256, 0, st>>>(x, w.dHpre, offsets, w.tok, s.Bs, s.d, dW1);
  }
  SPT_LAUNCH_CHECK();
  const dim3 g2(tiles, (s.d + TILE - 1) / TILE);
  {
    ScopedKernelTimer tm(kSlotDXPart, st);
    if (s.Bs <= TILE)
      kb_gemm_rows_kernel<<<tiles, 256, 0, st>>>(w1, w.dHpre, offsets, w.tile_prefix, s.N, s.Bs, s.d, w.part);
    else
      kb_gemm_kernel<<<g2, 256, 0, st>>>(w1, w.dHpre, offsets, w.tile_prefix, s.N, s.Bs, s.d, w.part);
  }
  SPT_LAUNCH_CHECK();
  return run_combine(s, w.part, inv, dX, kSlotCombineDX, st);
}

}  // namespace spt
