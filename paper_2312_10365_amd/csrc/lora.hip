// Low-rank adapted routed FFN (paper section 2.2: a projection Y = XW becomes X(W + BC) with W
// frozen; section 4.2 routing on top): the small kernels around the big GEMMs.
//
// With rank r <= 32 every adapter term is a product through a 32-wide bottleneck, so it is kept
// out of the big GEMMs' way instead of being merged into the weights:
//   inner projection   hpre += C1_b^T (A1^T x):  U = X A1 is computed once per token
//                      (lora_proj) and enters the K = d GEMM as 64 more K-values (each of the
//                      32 padded ranks as a bf16 value plus a bf16 remainder);
//   outer projection   y += C2^T (sum_b B2_b^T h_b): per pair Sp = H B2_b (lora_pair_gemm),
//                      summed per token (lora_token_sum), times C2 (lora_expand) as one more
//                      row for the combine to add;
//   backward           the transposes of the same three steps, and the adapter gradients as
//                      weight-gradient GEMMs with a 32-wide side (run by the dW kernel).
// All adapter operands are first copied into zero-padded bf16 panels with 32 in place of r
// (lora_pad), so no kernel below has a ragged rank dimension.
#include "ffn_common.hpp"
#include "spt_host.hpp"
#include "profile.hpp"

namespace spt {

// dst[a][b] (drows x dcols, bf16) = transpose ? src[b'][a] : src[a][b'] with b' = b, or b % 32
// when dup is set (a 32-wide panel repeated in columns 32..63); zero outside src (srows x scols).
// (Up to kMaxPadJobs panels per launch: blockIdx.y picks the job.)
__global__ void lora_pad_kernel(PadJobs jobs) {
  const PadJob j = jobs.job[blockIdx.y];
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= (int64_t)j.drows * j.dcols) return;
  const int a = (int)(id / j.dcols);
  int b = (int)(id % j.dcols);
  if (j.dup) b &= 31;
  const int sr = j.transpose ? b : a, sc = j.transpose ? a : b;
  j.dst[id] = (sr < j.srows && sc < j.scols) ? j.src[(size_t)sr * j.scols + sc] : (uint16_t)0;
}

// Z[t][c] = sum_rho S[t][rho] * MT[c][rho] (rho < 32), rounded to bf16: the low-rank term of an
// outer projection as one more "partial row" per token for the combine.  A wavefront takes 32
// tokens x 128 columns; the columns are the MFMA rows, through rho32, so a lane ends up with 16
// consecutive columns of one token.
__global__ __launch_bounds__(256) void lora_expand_kernel(const float* __restrict__ S,
                                                          const uint16_t* __restrict__ MT, int T, int d,
                                                          uint16_t* __restrict__ Z) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int i = lane & 31, h = lane >> 5;
  const int t0 = blockIdx.x * 32, c0 = (blockIdx.y * 4 + wave) * 128;
  if (c0 >= d) return;
  const int t = (t0 + i < T) ? t0 + i : T - 1;
  bf16x8 sb[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    const float* sp = S + (size_t)t * 32 + 16 * ks + 8 * h;
    const f32x4 lo = *reinterpret_cast<const f32x4*>(sp), hi = *reinterpret_cast<const f32x4*>(sp + 4);
    sb[ks] = as_bf16x8(make_uint4(pack_bf16x2(lo[0], lo[1]), pack_bf16x2(lo[2], lo[3]),
                                  pack_bf16x2(hi[0], hi[1]), pack_bf16x2(hi[2], hi[3])));
  }
#pragma unroll
  for (int ct = 0; ct < 4; ++ct) {
    const int c = c0 + ct * 32;
    if (c >= d) break;  // d is a multiple of 64, tiles are 32 wide: whole tiles only
    const uint16_t* mrow = MT + (size_t)(c + rho32(i)) * 32 + 8 * h;
    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
          as_bf16x8(*reinterpret_cast<const uint4*>(mrow + 16 * ks)), sb[ks], acc, 0, 0, 0);
    if (t0 + i < T) {
      uint4* dst = reinterpret_cast<uint4*>(Z + (size_t)(t0 + i) * d + c + 16 * h);
      dst[0] = make_uint4(pack_bf16x2(acc[0], acc[1]), pack_bf16x2(acc[2], acc[3]),
                          pack_bf16x2(acc[4], acc[5]), pack_bf16x2(acc[6], acc[7]));
      dst[1] = make_uint4(pack_bf16x2(acc[8], acc[9]), pack_bf16x2(acc[10], acc[11]),
                          pack_bf16x2(acc[12], acc[13]), pack_bf16x2(acc[14], acc[15]));
    }
  }
}

// S[t][rho] = sum_i Act[t][i] * MT[rho][i], rho < 32, written as TWO bf16 numbers: the rounded
// value in column rho and the rounded remainder in column 32 + rho of the 64-wide row, so the
// pair carries about 16 mantissa bits.  (With one bf16 the 2^-9 rounding of this term would be
// enough to flip the sign of pre-activations near zero, which ReLU's derivative turns into
// visible gradient errors.)  A workgroup owns 32
// tokens; its four wavefronts split d four ways (v_mfma_f32_32x32x16_bf16, both operands
// K-contiguous and read straight from global memory) and add their parts through LDS in wave
// order.
__global__ __launch_bounds__(256) void lora_proj_kernel(const uint16_t* __restrict__ Act,
                                                        const uint16_t* __restrict__ MT, int T, int d,
                                                        uint16_t* __restrict__ S) {
  __shared__ float red[4][32][33];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int i = lane & 31, h = lane >> 5;
  const int t0 = blockIdx.x * 32;
  const int t = (t0 + i < T) ? t0 + i : T - 1;  // clamped rows are computed but never stored
  const int kq = d / 4;                          // d is a multiple of 64: each part a multiple of 16
  const uint16_t* arow = Act + (size_t)t * d + wave * kq + 8 * h;
  const uint16_t* brow = MT + (size_t)i * d + wave * kq + 8 * h;
  f32x16 acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
  for (int k0 = 0; k0 < kq; k0 += 64) {
    uint4 a[4], b[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const bool ok = k0 + 16 * s < kq;
      a[s] = ok ? *reinterpret_cast<const uint4*>(arow + k0 + 16 * s) : make_uint4(0, 0, 0, 0);
      b[s] = ok ? *reinterpret_cast<const uint4*>(brow + k0 + 16 * s) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int s = 0; s < 4; ++s)
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a[s]), as_bf16x8(b[s]), acc, 0, 0, 0);
  }
  // C layout: lane (column rho = i, half h) holds token rows 8 g + 4 h + e in acc[4 g + e]
#pragma unroll
  for (int v = 0; v < 16; ++v) red[wave][8 * (v >> 2) + 4 * h + (v & 3)][i] = acc[v];
  __syncthreads();
  for (int e = tid; e < 32 * 32; e += 256) {
    const int row = e >> 5, rho = e & 31;
    if (t0 + row < T) {
      const float sum = ((red[0][row][rho] + red[1][row][rho]) + red[2][row][rho]) + red[3][row][rho];
      const uint32_t hi = f32_to_bf16_bits(sum);
      S[(size_t)(t0 + row) * 64 + rho] = (uint16_t)hi;
      S[(size_t)(t0 + row) * 64 + 32 + rho] = (uint16_t)f32_to_bf16_bits(sum - bf16_to_f32((uint16_t)hi));
    }
  }
}

// Per pair: Sp[q][rho] = sum_u f(Hin[q][u]) * WT[rho][b*Bs + u], b the bucket of sorted position
// q, f the activation (ACT 0 / 1) or the identity (ACT 2).  A workgroup takes 32 consecutive
// sorted positions and its four wavefronts a quarter of the block's hidden units each (added
// through LDS in wave order); where the 32 positions straddle buckets it makes one masked pass
// per bucket.
template <int ACT, bool FRAG>
__global__ __launch_bounds__(256) void lora_pair_gemm_kernel(const uint16_t* __restrict__ Hin,
                                                             const uint16_t* __restrict__ WT,
                                                             const int32_t* __restrict__ offsets, int N,
                                                             int Bs, int P, float* __restrict__ Sp) {
  __shared__ float red[3][64][17];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, i = lane & 31, h = lane >> 5;
  const int qbase = blockIdx.x * 32;
  const size_t D = (size_t)N * Bs;
  const int qstop = (qbase + 32 < P) ? qbase + 32 : P;
  const int per = ((Bs / 16 + 3) / 4) * 16;  // hidden units per wavefront, a multiple of 16
  const int ub = wave * per, ue = (ub + per < Bs) ? ub + per : Bs;
  int q = qbase;
  while (q < qstop) {
    int lo = 0, hi = N;  // the bucket of q: the largest b with offsets[b] <= q
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (offsets[mid] <= q) lo = mid; else hi = mid;
    }
    const int b = lo;
    const int qe = min(qstop, offsets[b + 1]);
    const int row = qbase + i;
    const bool mine = row >= q && row < qe;
    const int hq = mine ? row : q;
    const uint16_t* wrow = WT + (size_t)i * D + (size_t)b * Bs + 8 * h;
    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    for (int u0 = ub; u0 < ue; u0 += 16) {
      uint4 hv = *reinterpret_cast<const uint4*>(Hin + hval_off<FRAG>(hq, u0 + 8 * h, Bs));
      const uint4 wv = *reinterpret_cast<const uint4*>(wrow + u0);
      if (ACT != 2) {
        uint32_t* w = reinterpret_cast<uint32_t*>(&hv);
#pragma unroll
        for (int e = 0; e < 4; ++e)
          w[e] = pack_bf16x2(act_fn<(ACT & 1)>(lo_bf16(w[e])), act_fn<(ACT & 1)>(hi_bf16(w[e])));
      }
      // A operand: rows rho (WT), B operand: columns = sorted positions (Hin)
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(wv), as_bf16x8(hv), acc, 0, 0, 0);
    }
    __syncthreads();  // the previous pass has been read out
    if (wave > 0) {
#pragma unroll
      for (int v = 0; v < 16; ++v) red[wave - 1][lane][v] = acc[v];
    }
    __syncthreads();
    // lane (column = position i, half h) holds rho = 8 g + 4 h + e in acc[4 g + e]
    if (wave == 0 && mine) {
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[v] = ((acc[v] + red[0][lane][v]) + red[1][lane][v]) + red[2][lane][v];
#pragma unroll
      for (int g = 0; g < 4; ++g)
        *reinterpret_cast<f32x4*>(Sp + (size_t)row * 32 + 8 * g + 4 * h) =
            f32x4{acc[4 * g], acc[4 * g + 1], acc[4 * g + 2], acc[4 * g + 3]};
    }
    q = qe;
  }
}

// Per token: Sf[t][rho] = sum_j Sp[inv[t*k + j]][rho], j ascending; Sb (optional) the same
// rounded to bf16.  Eight gathered values are requested before the first is added.
__global__ void lora_token_sum_kernel(const float* __restrict__ Sp, const int32_t* __restrict__ inv,
                                      int T, int k, float* __restrict__ Sf, uint16_t* __restrict__ Sb) {
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= (int64_t)T * 32) return;
  const int t = (int)(id >> 5), rho = (int)(id & 31);
  const int32_t* iv = inv + (size_t)t * k;
  float s = 0.f;
  int j = 0;
  for (; j + 8 <= k; j += 8) {
    float v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = Sp[(size_t)iv[j + e] * 32 + rho];
#pragma unroll
    for (int e = 0; e < 8; ++e) s += v[e];
  }
  for (; j < k; ++j) s += Sp[(size_t)iv[j] * 32 + rho];
  if (Sf) Sf[id] = s;
  if (Sb) Sb[id] = (uint16_t)f32_to_bf16_bits(s);
}

// Identity schedule for the dW kernel run over ALL tokens in chunks: offsets[c] = min(c*chunk, T),
// tok[t] = t, border[c] = c.
__global__ void lora_chunks_kernel(int T, int chunk, int nchunks, int32_t* __restrict__ offsets,
                                   int32_t* __restrict__ tok, int32_t* __restrict__ border) {
  const int id = blockIdx.x * blockDim.x + threadIdx.x;
  if (id < T) tok[id] = id;
  if (id <= nchunks) offsets[id] = (int64_t)id * chunk < T ? id * chunk : T;
  if (id < nchunks) border[id] = id;
}

// Buckets cut into pieces of at most `piece` rows, so that the K = bucket rows adapter gradients
// run as many small GEMMs instead of a few long ones (with 4 or 8 wide blocks there are only 4 or
// 8 buckets).  One workgroup, thread b = bucket b: first[b] = index of b's first piece
// (first[N] = total), p_off[p] / p_off[p+1] = the row range of piece p; unused pieces up to
// max_pieces are empty ranges at the end.
__global__ __launch_bounds__(1024) void lora_pieces_kernel(const int32_t* __restrict__ offsets, int N,
                                                           int piece, int max_pieces,
                                                           int32_t* __restrict__ first,
                                                           int32_t* __restrict__ p_off,
                                                           int32_t* __restrict__ p_id) {
  __shared__ int32_t scan[1024];
  const int b = threadIdx.x;
  const int o0 = (b < N) ? offsets[b] : 0;
  const int m = (b < N) ? offsets[b + 1] - o0 : 0;
  const int np = (m + piece - 1) / piece;
  scan[b] = np;
  __syncthreads();
  for (int s = 1; s < 1024; s <<= 1) {
    const int t = (b >= s) ? scan[b - s] : 0;
    __syncthreads();
    scan[b] += t;
    __syncthreads();
  }
  const int begin = scan[b] - np;
  if (b < N) {
    first[b] = begin;
    for (int p = 0; p < np; ++p) p_off[begin + p] = o0 + p * piece;
  }
  const int total = scan[1023];
  const int last_row = offsets[N];
  if (b == 0) first[N] = total;
  for (int p = total + b; p <= max_pieces; p += 1024) p_off[p] = last_row;
  for (int p = b; p < max_pieces; p += 1024) p_id[p] = p;
}

// out (fp32) from per-piece results src[piece][Bs][64]: for hidden unit (b, u) and rank rho,
// sum over b's pieces (in order) of src[.][u][rho] + src[.][u][rho + 32]; written as
// out[rho][b*Bs+u] (transpose) or out[b*Bs+u][rho].
__global__ void lora_reduce_pieces_kernel(const float* __restrict__ src, const int32_t* __restrict__ first,
                                          int N, int Bs, int r, int transpose, float* __restrict__ out) {
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t D = (int64_t)N * Bs;
  if (id >= D * 32) return;
  const int rho = (int)(id & 31);
  const int64_t unit = id >> 5;
  if (rho >= r) return;
  const int b = (int)(unit / Bs), u = (int)(unit % Bs);
  float s = 0.f;
  for (int p = first[b]; p < first[b + 1]; ++p) {
    const float* row = src + ((size_t)p * Bs + u) * 64;
    s += row[rho] + row[rho + 32];
  }
  if (transpose) out[(size_t)rho * D + unit] = s;
  else out[(size_t)unit * r + rho] = s;
}

// out[a][b] (orows x ocols, fp32) = sum_c src[c][.][.] taken in chunk order, where one chunk of
// src is a (srows x scols) matrix and (a, b) maps to (b, a) when transpose is set.  With fold
// set, source column sc + 32 (the product with the remainder halves of a two-part panel) is
// added to source column sc.
__global__ void lora_reduce_kernel(const float* __restrict__ src, int nchunks, int srows, int scols,
                                   int transpose, int fold, float* __restrict__ out, int orows,
                                   int ocols) {
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= (int64_t)orows * ocols) return;
  const int a = (int)(id / ocols), b = (int)(id % ocols);
  const int sr = transpose ? b : a, sc = transpose ? a : b;
  const size_t stride = (size_t)srows * scols;
  float s = 0.f;
  for (int c = 0; c < nchunks; ++c) {
    const float* row = src + (size_t)c * stride + (size_t)sr * scols;
    s += fold ? row[sc] + row[sc + 32] : row[sc];
  }
  out[id] = s;
}

#define SPT_LAUNCH_CHECK()                 \
  do {                                     \
    hipError_t e_ = hipGetLastError();     \
    if (e_ != hipSuccess) return e_;       \
  } while (0)

hipError_t lora_pad(const PadJobs& jobs, int njobs, hipStream_t st) {
  int64_t n = 0;
  for (int j = 0; j < njobs; ++j) {
    const int64_t m = (int64_t)jobs.job[j].drows * jobs.job[j].dcols;
    if (m > n) n = m;
  }
  lora_pad_kernel<<<dim3((unsigned)((n + 255) / 256), njobs), 256, 0, st>>>(jobs);
  SPT_LAUNCH_CHECK();
  return hipSuccess;
}

hipError_t lora_expand(const float* S, const uint16_t* MT, int T, int d, uint16_t* Z, hipStream_t st) {
  lora_expand_kernel<<<dim3((T + 31) / 32, (d + 511) / 512), 256, 0, st>>>(S, MT, T, d, Z);
  SPT_LAUNCH_CHECK();
  return hipSuccess;
}

hipError_t lora_proj(const uint16_t* Act, const uint16_t* MT, int T, int d, uint16_t* S, hipStream_t st) {
  lora_proj_kernel<<<(T + 31) / 32, 256, 0, st>>>(Act, MT, T, d, S);
  SPT_LAUNCH_CHECK();
  return hipSuccess;
}

hipError_t lora_pair_gemm(const uint16_t* Hin, bool hin_frag, const uint16_t* WT, const int32_t* offsets, int N,
                          int Bs, int P, int act, float* Sp, hipStream_t st) {
  const unsigned grid = (unsigned)(((int64_t)P + 31) / 32);
  if (act == 0) lora_pair_gemm_kernel<0, false><<<grid, 256, 0, st>>>(Hin, WT, offsets, N, Bs, P, Sp);
  else if (act == 1) lora_pair_gemm_kernel<1, false><<<grid, 256, 0, st>>>(Hin, WT, offsets, N, Bs, P, Sp);
  else if (hin_frag) lora_pair_gemm_kernel<2, true><<<grid, 256, 0, st>>>(Hin, WT, offsets, N, Bs, P, Sp);
  else lora_pair_gemm_kernel<2, false><<<grid, 256, 0, st>>>(Hin, WT, offsets, N, Bs, P, Sp);
  SPT_LAUNCH_CHECK();
  return hipSuccess;
}

hipError_t lora_token_sum(const float* Sp, const int32_t* inv, int T, int k, float* Sf, uint16_t* Sb,
                          hipStream_t st) {
  const int64_t n = (int64_t)T * 32;
  lora_token_sum_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(Sp, inv, T, k, Sf, Sb);
  SPT_LAUNCH_CHECK();
  return hipSuccess;
}

hipError_t lora_chunks(int T, int chunk, int nchunks, int32_t* offsets, int32_t* tok, int32_t* border,
                       hipStream_t st) {
  const int n = T > nchunks + 1 ? T : nchunks + 1;
  lora_chunks_kernel<<<(n + 255) / 256, 256, 0, st>>>(T, chunk, nchunks, offsets, tok, border);
  SPT_LAUNCH_CHECK();
  return hipSuccess;
}

hipError_t lora_pieces(const int32_t* offsets, int N, int piece, int max_pieces, int32_t* first,
                       int32_t* p_off, int32_t* p_id, hipStream_t st) {
  lora_pieces_kernel<<<1, 1024, 0, st>>>(offsets, N, piece, max_pieces, first, p_off, p_id);
  SPT_LAUNCH_CHECK();
  return hipSuccess;
}

hipError_t lora_reduce_pieces(const float* src, const int32_t* first, int N, int Bs, int r, bool transpose,
                              float* out, hipStream_t st) {
  const int64_t n = (int64_t)N * Bs * 32;
  lora_reduce_pieces_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(src, first, N, Bs, r,
                                                                         transpose ? 1 : 0, out);
  SPT_LAUNCH_CHECK();
  return hipSuccess;
}

hipError_t lora_reduce(const float* src, int nchunks, int srows, int scols, bool transpose, bool fold,
                       float* out, int orows, int ocols, hipStream_t st) {
  const int64_t n = (int64_t)orows * ocols;
  lora_reduce_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(
      src, nchunks, srows, scols, transpose ? 1 : 0, fold ? 1 : 0, out, orows, ocols);
  SPT_LAUNCH_CHECK();
  return hipSuccess;
}

}  // namespace spt
