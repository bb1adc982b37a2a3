// Route network + block selection (paper section 4.2, "Dynamic routing").
//
// logit[t][b] = sum_i X[t][i] * W_r[i][b] (+ b_r[b]) accumulated in fp64 and rounded once to
// fp32.  Products of a bf16 and an fp32 value are exact in fp64, so only the order of the
// additions can move the fp64 sum, by parts in 1e-16 -- far below the fp32 rounding step.
// The k largest keys win; equal keys go to the lower block id; ids are emitted ascending.
//
// Kernel 1 (logits): fp64 matrix cores, v_mfma_f64_16x16x4_f64.  A workgroup of 4 wavefronts
// owns 64 tokens x 64 blocks, each wavefront a 32 x 32 quadrant (2 x 2 MFMA tiles) over the
// whole of d.  Operands go straight from global memory to registers: a lane reads 8
// consecutive bf16 of one token row and the matching 8 rows of one W_r column, widens them to
// fp64, and feeds 8 MFMAs; which real k sits in which MFMA k-slot is the same for both
// operands, which is all a contraction needs.
// Kernel 2 (top-k): one wavefront per token, rank-by-counting over the fp32 keys:
// rank(b) = #{b' : key[b'] > key[b] or (key[b'] == key[b] and b' < b)}; selected iff rank < k.
#include "spt_device.hpp"
#include "spt_host.hpp"
#include "profile.hpp"

namespace spt {

typedef double f64x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void router_logits_kernel(
    const uint16_t* __restrict__ X, const float* __restrict__ Wr, const float* __restrict__ br,
    int T, int d, int N, float* __restrict__ logits) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r16 = lane & 15, slot = lane >> 4;
  const int tok0 = blockIdx.x * 64 + (wave >> 1) * 32;
  const int blk0 = blockIdx.y * 64 + (wave & 1) * 32;

  const uint16_t* xrow[2];
  const float* wcol[2];
  bool bok[2];
#pragma unroll
  for (int m = 0; m < 2; ++m) {
    const int t = min(tok0 + 16 * m + r16, T - 1);  // clamped rows are computed but never stored
    xrow[m] = X + (size_t)t * d + 8 * slot;
    const int b = blk0 + 16 * m + r16;
    bok[m] = b < N;
    wcol[m] = Wr + (size_t)(8 * slot) * N + (bok[m] ? b : 0);
  }
  f64x4 acc[2][2];
#pragma unroll
  for (int m = 0; m < 2; ++m)
#pragma unroll
    for (int n = 0; n < 2; ++n) acc[m][n] = f64x4{0.0, 0.0, 0.0, 0.0};

  uint4 xa[2], xn[2];
  float wb[2][8], wn[2][8];
#pragma unroll
  for (int m = 0; m < 2; ++m) {
    xa[m] = *reinterpret_cast<const uint4*>(xrow[m]);
#pragma unroll
    for (int e = 0; e < 8; ++e) wb[m][e] = wcol[m][(size_t)e * N];
  }
  for (int k0 = 0; k0 < d; k0 += 32) {
    const bool more = k0 + 32 < d;
    if (more) {
#pragma unroll
      for (int m = 0; m < 2; ++m) {
        xn[m] = *reinterpret_cast<const uint4*>(xrow[m] + k0 + 32);
#pragma unroll
        for (int e = 0; e < 8; ++e) wn[m][e] = wcol[m][(size_t)(k0 + 32 + e) * N];
      }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      double a[2], b[2];
#pragma unroll
      for (int m = 0; m < 2; ++m) {
        const uint32_t w32 = reinterpret_cast<const uint32_t*>(&xa[m])[e >> 1];
        a[m] = (double)((e & 1) ? hi_bf16(w32) : lo_bf16(w32));
        b[m] = bok[m] ? (double)wb[m][e] : 0.0;
      }
#pragma unroll
      for (int m = 0; m < 2; ++m)
#pragma unroll
        for (int n = 0; n < 2; ++n)
          acc[m][n] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[m], b[n], acc[m][n], 0, 0, 0);
    }
    if (more) {
#pragma unroll
      for (int m = 0; m < 2; ++m) {
        xa[m] = xn[m];
#pragma unroll
        for (int e = 0; e < 8; ++e) wb[m][e] = wn[m][e];
      }
    }
  }
  // D layout of the 16x16 fp64 tile: lane holds column (lane & 15), rows 4*v + (lane >> 4).
#pragma unroll
  for (int m = 0; m < 2; ++m)
#pragma unroll
    for (int n = 0; n < 2; ++n) {
      const int b = blk0 + 16 * n + r16;
      if (b >= N) continue;
      const double bias = br ? (double)br[b] : 0.0;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int t = tok0 + 16 * m + 4 * v + slot;
        if (t < T) logits[(size_t)t * N + b] = (float)(acc[m][n][v] + bias);
      }
    }
}

template <int NPL>
__global__ __launch_bounds__(256) void topk_kernel(const float* __restrict__ logits, int T, int N,
                                                   int k, int flags, int32_t* __restrict__ idx) {
  __shared__ float keys[4][NPL * 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int t_raw = blockIdx.x * 4 + wave;
  const bool live = t_raw < T;
  const int t = live ? t_raw : T - 1;  // surplus wavefronts redo the last token, store nothing
  float* krow = keys[wave];
  float mykey[NPL];
  int rank[NPL];
#pragma unroll
  for (int n = 0; n < NPL; ++n) {
    const int b = lane + 64 * n;
    float key = -INFINITY;
    if (b < N) {
      const float l = logits[(size_t)t * N + b];
      key = (flags & 1) ? fabsf(l) : l;
    }
    mykey[n] = key;
    krow[b] = key;
    rank[n] = 0;
  }
  __syncthreads();
  for (int bp = 0; bp < N; ++bp) {
    const float kb = krow[bp];
#pragma unroll
    for (int n = 0; n < NPL; ++n) {
      const int b = lane + 64 * n;
      rank[n] += (kb > mykey[n]) || (kb == mykey[n] && bp < b);
    }
  }
  int base = 0;
#pragma unroll
  for (int n = 0; n < NPL; ++n) {
    const int b = lane + 64 * n;
    const bool sel = (b < N) && (rank[n] < k);
    const unsigned long long m = __ballot(sel);
    const int pos = base + __popcll(m & ((1ull << lane) - 1ull));
    if (sel && live) idx[(size_t)t * k + pos] = b;
    base += __popcll(m);
  }
}

template <int NPL>
static void launch_topk(const spt_shape_t& s, const float* logits, int32_t* idx, hipStream_t st) {
  topk_kernel<NPL><<<(s.T + 3) / 4, 256, 0, st>>>(logits, s.T, s.N, s.k, s.flags, idx);
}

hipError_t run_router_topk(const spt_shape_t& s, const void* X, const float* Wr, const float* br,
                           int32_t* idx, float* logits, hipStream_t st) {
  {
    ScopedKernelTimer tm(kSlotRouter, st);
    const dim3 grid((s.T + 63) / 64, (s.N + 63) / 64);
    router_logits_kernel<<<grid, 256, 0, st>>>(static_cast<const uint16_t*>(X), Wr, br, s.T, s.d,
                                               s.N, logits);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  {
    ScopedKernelTimer tm(kSlotTopk, st);
    const int npl = (s.N + 63) / 64;
    if (npl <= 1) launch_topk<1>(s, logits, idx, st);
    else if (npl <= 2) launch_topk<2>(s, logits, idx, st);
    else if (npl <= 4) launch_topk<4>(s, logits, idx, st);
    else if (npl <= 8) launch_topk<8>(s, logits, idx, st);
    else launch_topk<16>(s, logits, idx, st);
  }
  return hipGetLastError();
}

}  // namespace spt
