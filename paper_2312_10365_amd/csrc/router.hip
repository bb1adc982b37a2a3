// Route network + block selection (paper section 4.2, "Dynamic routing").
//
// logit[t][b] = sum_i X[t][i] * W_r[i][b] (+ b_r[b]), summed in fp64 with i ascending and
// rounded once to fp32.  Products of a bf16 and an fp32 value are exact in fp64, so the sum
// depends only on the order, which is fixed.  The k largest keys win; equal keys go to the
// lower block id; ids are emitted ascending.
//
// One workgroup = 4 wavefronts = 32 tokens (8 per wavefront).  Lane l of a wavefront owns
// blocks l, l+64, ...; a chunk of W_r rows and of the 32 token rows is widened to fp64 in
// LDS once and then streamed through fp64 FMAs.  Selection is rank-by-counting inside the
// wavefront: rank(b) = #{b' : key[b'] > key[b] or (key[b'] == key[b] and b' < b)}.
#include "spt_device.hpp"
#include "spt_host.hpp"
#include "profile.hpp"

namespace spt {

constexpr int kRouterTokPerWG = 32;
constexpr int kRouterTokPerWave = 8;
constexpr int kXsPitch = 33;  // doubles per staged X row: odd pitch keeps LDS writes conflict-free

template <int NPL>
__global__ __launch_bounds__(256) void router_topk_kernel(
    const uint16_t* __restrict__ X, const float* __restrict__ Wr, const float* __restrict__ br,
    int T, int d, int N, int k, int flags, int ic_log2, int32_t* __restrict__ idx,
    float* __restrict__ logits) {
  extern __shared__ double smem[];
  constexpr int Npad = NPL * 64;
  const int IC = 1 << ic_log2;
  double* Wd = smem;                       // [IC][Npad]
  double* xs = smem + (size_t)IC * Npad;   // [IC][kXsPitch]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int t0 = blockIdx.x * kRouterTokPerWG;

  double acc[kRouterTokPerWave][NPL];
#pragma unroll
  for (int a = 0; a < kRouterTokPerWave; ++a)
#pragma unroll
    for (int n = 0; n < NPL; ++n) acc[a][n] = 0.0;

  for (int i0 = 0; i0 < d; i0 += IC) {
    __syncthreads();
    for (int e = tid; e < IC * Npad; e += 256) {
      const int ii = e / Npad, b = e % Npad;
      Wd[e] = (b < N) ? (double)Wr[(size_t)(i0 + ii) * N + b] : 0.0;
    }
    for (int e = tid; e < kRouterTokPerWG * IC; e += 256) {
      const int tk = e >> ic_log2, ii = e & (IC - 1);
      const int t = t0 + tk;
      xs[ii * kXsPitch + tk] = (t < T) ? (double)bf16_to_f32(X[(size_t)t * d + i0 + ii]) : 0.0;
    }
    __syncthreads();
    for (int ii = 0; ii < IC; ++ii) {
      double w[NPL];
#pragma unroll
      for (int n = 0; n < NPL; ++n) w[n] = Wd[ii * Npad + lane + 64 * n];
      const double* xr = xs + ii * kXsPitch + wave * kRouterTokPerWave;
#pragma unroll
      for (int a = 0; a < kRouterTokPerWave; ++a) {
        const double x = xr[a];
#pragma unroll
        for (int n = 0; n < NPL; ++n) acc[a][n] = fma(x, w[n], acc[a][n]);
      }
    }
  }
  __syncthreads();

  float* keys = reinterpret_cast<float*>(smem);  // [32][Npad]
#pragma unroll
  for (int a = 0; a < kRouterTokPerWave; ++a) {
    const int t = t0 + wave * kRouterTokPerWave + a;
#pragma unroll
    for (int n = 0; n < NPL; ++n) {
      const int b = lane + 64 * n;
      float key = -INFINITY;
      if (b < N) {
        const double v = acc[a][n] + (br ? (double)br[b] : 0.0);
        const float l = (float)v;
        if (logits && t < T) logits[(size_t)t * N + b] = l;
        key = (flags & 1) ? fabsf(l) : l;
      }
      keys[(wave * kRouterTokPerWave + a) * Npad + b] = key;
    }
  }
  __syncthreads();

  for (int a = 0; a < kRouterTokPerWave; ++a) {
    const int t = t0 + wave * kRouterTokPerWave + a;
    if (t >= T) break;
    const float* krow = keys + (wave * kRouterTokPerWave + a) * Npad;
    float mykey[NPL];
    int rank[NPL];
#pragma unroll
    for (int n = 0; n < NPL; ++n) {
      mykey[n] = krow[lane + 64 * n];
      rank[n] = 0;
    }
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
      if (sel) idx[(size_t)t * k + pos] = b;
      base += __popcll(m);
    }
  }
}

static int router_ic_log2(int npl) {
  // W_r chunk in LDS: IC * Npad doubles <= 64 KiB.
  int ic = 8192 / (npl * 64);
  if (ic > 64) ic = 64;
  int lg = 0;
  while ((1 << (lg + 1)) <= ic) ++lg;
  return lg;
}

template <int NPL>
static hipError_t launch_router(const spt_shape_t& s, const void* X, const float* Wr,
                                const float* br, int32_t* idx, float* logits, hipStream_t st) {
  const int lg = router_ic_log2(NPL);
  const int IC = 1 << lg;
  size_t smem = ((size_t)IC * NPL * 64 + (size_t)IC * kXsPitch) * sizeof(double);
  const size_t keys = (size_t)kRouterTokPerWG * NPL * 64 * sizeof(float);
  if (keys > smem) smem = keys;
  const int grid = (s.T + kRouterTokPerWG - 1) / kRouterTokPerWG;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(router_topk_kernel<NPL>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (e != hipSuccess) return e;
  {
    ScopedKernelTimer tm(kSlotRouter, st);
    router_topk_kernel<NPL><<<grid, 256, smem, st>>>(static_cast<const uint16_t*>(X), Wr, br, s.T,
                                                      s.d, s.N, s.k, s.flags, lg, idx, logits);
  }
  return hipGetLastError();
}

hipError_t run_router_topk(const spt_shape_t& s, const void* X, const float* Wr, const float* br,
                           int32_t* idx, float* logits, hipStream_t st) {
  const int npl = (s.N + 63) / 64;
  if (npl <= 1) return launch_router<1>(s, X, Wr, br, idx, logits, st);
  if (npl <= 2) return launch_router<2>(s, X, Wr, br, idx, logits, st);
  if (npl <= 4) return launch_router<4>(s, X, Wr, br, idx, logits, st);
  if (npl <= 8) return launch_router<8>(s, X, Wr, br, idx, logits, st);
  return launch_router<16>(s, X, Wr, br, idx, logits, st);
}

}  // namespace spt
