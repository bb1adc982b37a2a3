// Route network + block selection (paper section 4.2, "Dynamic routing").
//
// logit[t][b] = sum_i X[t][i] * W_r[i][b] (+ b_r[b]) accumulated in fp64 and rounded once to
// fp32.  Products of a bf16 and an fp32 value are exact in fp64, so only the order of the
// additions can move the fp64 sum, by parts in 1e-16 -- far below the fp32 rounding step.
// The k largest keys win; equal keys go to the lower block id; ids are emitted ascending.
//
// Kernel 1 (logits): fp64 matrix cores, v_mfma_f64_16x16x4_f64.  A workgroup of 4 wavefronts
// owns 64 tokens x 32 blocks, each wavefront a 32 x 16 part (2 MFMA tiles) over the whole of d.
// Operands go straight from global memory to registers: a lane reads 8
// consecutive bf16 of one token row and the matching 8 rows of one W_r column, widens them to
// fp64, and feeds 8 MFMAs; which real k sits in which MFMA k-slot is the same for both
// operands, which is all a contraction needs.
// Kernel 2 (top-k): one wavefront per token; the k-th largest key is found by a 32-step radix
// search on the order-preserving integer image of the fp32 keys, the keys above it are selected,
// ties at it go to the lowest block ids: block b is selected iff fewer than k blocks b' have
// key[b'] > key[b] or (key[b'] == key[b] and b' < b).
#include "spt_device.hpp"
#include "spt_host.hpp"
#include "profile.hpp"

namespace spt {

typedef double f64x4 __attribute__((ext_vector_type(4)));

// NT = MFMA tiles per wavefront along the block axis: a wavefront owns 32 tokens x 16*NT
// blocks, a workgroup (2 x 2 wavefronts) 64 tokens x 32*NT blocks.  NT = 1 doubles the number
// of wavefronts per SIMD over NT = 2, which is what hides the global-load latency here: the
// operands are loaded two 32-wide k-chunks ahead of the MFMAs that consume them.
template <int NT, int KSPLIT>
__global__ __launch_bounds__(256 * KSPLIT) void router_logits_kernel(
    const uint16_t* __restrict__ X, const float* __restrict__ Wr, const float* __restrict__ br,
    int T, int d, int N, float* __restrict__ logits) {
  const int tid = threadIdx.x, lane = tid & 63, wave = (tid >> 6) & 3, kpart = tid >> 8;
  const int r16 = lane & 15, slot = lane >> 4;
  const int tok0 = blockIdx.x * 64 + (wave >> 1) * 32;
  const int blk0 = blockIdx.y * (32 * NT) + (wave & 1) * (16 * NT);
  const int kbeg = kpart * (d / KSPLIT);  // d is a multiple of 64: each part a multiple of 32

  const uint16_t* xrow[2];
  const float* wcol[NT];
  bool bok[NT];
#pragma unroll
  for (int m = 0; m < 2; ++m) {
    const int t = min(tok0 + 16 * m + r16, T - 1);  // clamped rows are computed but never stored
    xrow[m] = X + (size_t)t * d + kbeg + 8 * slot;
  }
#pragma unroll
  for (int n = 0; n < NT; ++n) {
    const int b = blk0 + 16 * n + r16;
    bok[n] = b < N;
    wcol[n] = Wr + (size_t)(kbeg + 8 * slot) * N + (bok[n] ? b : 0);
  }
  f64x4 acc[2][NT];
#pragma unroll
  for (int m = 0; m < 2; ++m)
#pragma unroll
    for (int n = 0; n < NT; ++n) acc[m][n] = f64x4{0.0, 0.0, 0.0, 0.0};

  // Register ring of three k-chunks: chunk c is consumed while c+1 and c+2 are in flight.
  uint4 xq[3][2];
  float wq[3][NT][8];
  auto fetch = [&](int st, int k0) {
#pragma unroll
    for (int m = 0; m < 2; ++m) xq[st][m] = *reinterpret_cast<const uint4*>(xrow[m] + k0);
#pragma unroll
    for (int n = 0; n < NT; ++n)
#pragma unroll
      for (int e = 0; e < 8; ++e) wq[st][n][e] = wcol[n][(size_t)(k0 + e) * N];
  };
  auto consume = [&](int st) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      double a[2], b[NT];
#pragma unroll
      for (int m = 0; m < 2; ++m) {
        const uint32_t w32 = reinterpret_cast<const uint32_t*>(&xq[st][m])[e >> 1];
        a[m] = (double)((e & 1) ? hi_bf16(w32) : lo_bf16(w32));
      }
#pragma unroll
      for (int n = 0; n < NT; ++n) b[n] = bok[n] ? (double)wq[st][n][e] : 0.0;
#pragma unroll
      for (int m = 0; m < 2; ++m)
#pragma unroll
        for (int n = 0; n < NT; ++n)
          acc[m][n] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[m], b[n], acc[m][n], 0, 0, 0);
    }
  };
  const int chunks = d / (32 * KSPLIT);
  fetch(0, 0);
  if (chunks > 1) fetch(1, 32);
  int c = 0;
  for (; c + 3 <= chunks; c += 3) {  // three chunks per trip keeps the ring slots static
    if (c + 2 < chunks) fetch(2, (c + 2) * 32);
    consume(0);
    if (c + 3 < chunks) fetch(0, (c + 3) * 32);
    consume(1);
    if (c + 4 < chunks) fetch(1, (c + 4) * 32);
    consume(2);
  }
  // chunks % 3 leftovers: ring slots 0 and 1 already hold them
  if (c < chunks) consume(0);
  if (c + 1 < chunks) consume(1);

  if (KSPLIT > 1) {  // sum the k-parts through LDS, in part order, into part 0
    __shared__ double red[(KSPLIT - 1) * 4 * 2 * NT * 4 * 64];
    if (kpart > 0) {
#pragma unroll
      for (int m = 0; m < 2; ++m)
#pragma unroll
        for (int n = 0; n < NT; ++n)
#pragma unroll
          for (int v = 0; v < 4; ++v)
            red[((((kpart - 1) * 4 + wave) * 2 + m) * NT + n) * 256 + v * 64 + lane] = acc[m][n][v];
    }
    __syncthreads();
    if (kpart > 0) return;
#pragma unroll
    for (int p = 1; p < KSPLIT; ++p)
#pragma unroll
      for (int m = 0; m < 2; ++m)
#pragma unroll
        for (int n = 0; n < NT; ++n)
#pragma unroll
          for (int v = 0; v < 4; ++v)
            acc[m][n][v] += red[((((p - 1) * 4 + wave) * 2 + m) * NT + n) * 256 + v * 64 + lane];
  }

  // D layout of the 16x16 fp64 tile: lane holds column (lane & 15), rows 4*v + (lane >> 4).
#pragma unroll
  for (int m = 0; m < 2; ++m)
#pragma unroll
    for (int n = 0; n < NT; ++n) {
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

// One wavefront per token, NPL keys per lane (block b = lane + 64 n).  The k-th largest key is
// found by a radix search on the order-preserving integer image of the fp32 keys (32 steps of
// compare + ballot + popcount: the largest T with at least k keys >= T); every key above it is
// selected, and of the keys equal to it the lowest block ids, as many as are still missing.  Ids
// are emitted ascending.  (Rank-by-counting, the first version, compared every key with every
// other: 1400 instructions per token at N = 128 against about 250.)
template <int NPL>
__global__ __launch_bounds__(256) void topk_kernel(const float* __restrict__ logits, int T, int N,
                                                   int k, int flags, int32_t* __restrict__ idx) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int t = blockIdx.x * 4 + wave;
  if (t >= T) return;                      // whole wavefront; the kernel has no barrier
  uint32_t u[NPL];                         // larger key <=> larger u; 0 for lanes past N (below every real key)
#pragma unroll
  for (int n = 0; n < NPL; ++n) {
    const int b = lane + 64 * n;
    u[n] = 0u;
    if (b < N) {
      const float l = logits[(size_t)t * N + b];
      const float key = ((flags & 1) ? fabsf(l) : l) + 0.0f;       // -0 -> +0: equal keys, equal images
      const uint32_t bits = __float_as_uint(key);
      u[n] = (bits & 0x80000000u) ? ~bits : (bits | 0x80000000u);
      if (u[n] == 0u) u[n] = 1u;           // (only a NaN with all mantissa bits set maps to 0)
    }
  }
  uint32_t thr = 0u;
#pragma unroll 1
  for (int bit = 31; bit >= 0; --bit) {
    const uint32_t cand = thr | (1u << bit);
    int c = 0;
#pragma unroll
    for (int n = 0; n < NPL; ++n) c += __popcll(__ballot(u[n] >= cand));
    if (c >= k) thr = cand;                // uniform
  }
  int above = 0;
#pragma unroll
  for (int n = 0; n < NPL; ++n) above += __popcll(__ballot(u[n] > thr));
  int need = k - above;                    // keys equal to the threshold still to take, lowest ids first
  int base = 0;
#pragma unroll
  for (int n = 0; n < NPL; ++n) {
    const int b = lane + 64 * n;
    const unsigned long long below = (1ull << lane) - 1ull;
    const unsigned long long eq = __ballot(u[n] == thr);
    const bool sel = (u[n] > thr) || (u[n] == thr && __popcll(eq & below) < need);
    need -= min(need, __popcll(eq));
    const unsigned long long m = __ballot(sel);
    const int pos = base + __popcll(m & below);
    if (sel) idx[(size_t)t * k + pos] = b;
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
    // Two 16-block MFMA tiles per wavefront when there are blocks to fill them: the fp64
    // conversions of a token's values are then shared by both (they cost as much VALU time as the
    // MFMAs take), 0.159 against 0.168 ms at N = 128.
    if (s.N > 32) {
      const dim3 grid((s.T + 63) / 64, (s.N + 63) / 64);
      router_logits_kernel<2, 2><<<grid, 512, 0, st>>>(static_cast<const uint16_t*>(X), Wr, br, s.T, s.d, s.N,
                                                       logits);
    } else {
      const dim3 grid((s.T + 63) / 64, (s.N + 31) / 32);
      router_logits_kernel<1, 2><<<grid, 512, 0, st>>>(static_cast<const uint16_t*>(X), Wr, br, s.T, s.d, s.N,
                                                       logits);
    }
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

// ------------------------------------------------------------------------------------------
// Load-balancing loss of the route network (section 4.2 names such a loss; the formula is this
// build's choice, the usual one for top-k routers):
//   f_b = share of the (token, slot) pairs routed to block b (from the bucket offsets, held constant),
//   p_t = softmax of the token's logits, pbar_b = mean_t p_t[b],  loss = N sum_b f_b pbar_b,
//   dlogit[t][c] = (N / T) p_t[c] (f_c - sum_b f_b p_t[b]),  dW_r = X^T dlogit,  db_r = sum_t dlogit[t].
// Kernel 1: one wavefront per token (32 tokens in a row per wavefront), softmax in fp32; writes
// dlogit as bf16 rows padded to a multiple of 32 blocks (the operand of the dW_r GEMM) and, per
// workgroup, the sums of p and dlogit over its 128 tokens (added up in kernel 2 in group order).
constexpr int kBalTokPerWave = 32;

template <int NPL>
__global__ __launch_bounds__(256) void balance_kernel(const float* __restrict__ logits,
                                                      const int32_t* __restrict__ offsets, int T, int N,
                                                      int k, int npad, uint16_t* __restrict__ dl,
                                                      float* __restrict__ part,
                                                      uint32_t* __restrict__ zero_row) {
  __shared__ float red[3][2][NPL * 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (blockIdx.x == 0 && threadIdx.x < 64) zero_row[threadIdx.x] = 0u;
  float f[NPL], sp[NPL], sd[NPL];
  const float inv_pairs = 1.0f / ((float)T * (float)k);
#pragma unroll
  for (int n = 0; n < NPL; ++n) {
    const int b = lane + 64 * n;
    f[n] = (b < N) ? (float)(offsets[b + 1] - offsets[b]) * inv_pairs : 0.f;
    sp[n] = 0.f;
    sd[n] = 0.f;
  }
  const float scale = (float)N / (float)T;
  const int t0 = (blockIdx.x * 4 + wave) * kBalTokPerWave;
  for (int i = 0; i < kBalTokPerWave; ++i) {
    const int t = t0 + i;
    if (t >= T) break;  // wave-uniform
    float x[NPL];
    float m = -INFINITY;
#pragma unroll
    for (int n = 0; n < NPL; ++n) {
      const int b = lane + 64 * n;
      x[n] = (b < N) ? logits[(size_t)t * N + b] : -INFINITY;
      m = fmaxf(m, x[n]);
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    float ssum = 0.f;
#pragma unroll
    for (int n = 0; n < NPL; ++n) {
      x[n] = (lane + 64 * n < N) ? __expf(x[n] - m) : 0.f;
      ssum += x[n];
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) ssum += __shfl_xor(ssum, o);
    const float inv = 1.0f / ssum;
    float c = 0.f;
#pragma unroll
    for (int n = 0; n < NPL; ++n) {
      x[n] *= inv;  // p_t[b]
      c += f[n] * x[n];
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) c += __shfl_xor(c, o);
#pragma unroll
    for (int n = 0; n < NPL; ++n) {
      const int b = lane + 64 * n;
      const float g = scale * x[n] * (f[n] - c);
      sp[n] += x[n];
      sd[n] += g;
      if (b < npad) dl[(size_t)t * npad + b] = (uint16_t)f32_to_bf16_bits(b < N ? g : 0.f);
    }
  }
  if (wave > 0) {
#pragma unroll
    for (int n = 0; n < NPL; ++n) {
      red[wave - 1][0][lane + 64 * n] = sp[n];
      red[wave - 1][1][lane + 64 * n] = sd[n];
    }
  }
  __syncthreads();
  if (wave == 0) {
#pragma unroll
    for (int n = 0; n < NPL; ++n) {
      const int b = lane + 64 * n;
      if (b >= N) continue;
      const float p3 = ((sp[n] + red[0][0][b]) + red[1][0][b]) + red[2][0][b];
      const float d3 = ((sd[n] + red[0][1][b]) + red[1][1][b]) + red[2][1][b];
      part[((size_t)blockIdx.x * 2 + 0) * N + b] = p3;
      part[((size_t)blockIdx.x * 2 + 1) * N + b] = d3;
    }
  }
}

// Kernel 2 (one workgroup): pbar, db_r, the block shares and the loss, summed in fixed order.
__global__ __launch_bounds__(1024) void balance_reduce_kernel(const float* __restrict__ part,
                                                              const int32_t* __restrict__ offsets,
                                                              int groups, int T, int N, int k,
                                                              float* __restrict__ loss,
                                                              float* __restrict__ frac,
                                                              float* __restrict__ dbr) {
  __shared__ float term[1024];
  const int b = threadIdx.x;
  float sp = 0.f, sd = 0.f, fb = 0.f;
  if (b < N) {
    for (int g = 0; g < groups; ++g) {
      sp += part[((size_t)g * 2 + 0) * N + b];
      sd += part[((size_t)g * 2 + 1) * N + b];
    }
    fb = (float)(offsets[b + 1] - offsets[b]) / ((float)T * (float)k);
    if (frac) frac[b] = fb;
    if (dbr) dbr[b] = sd;
  }
  term[b] = (b < N) ? fb * (sp / (float)T) : 0.f;
  __syncthreads();
  if (b == 0) {
    float s = 0.f;
    for (int c = 0; c < N; ++c) s += term[c];
    *loss = (float)N * s;
  }
}

template <int NPL>
static void launch_balance(const float* logits, const int32_t* offsets, const spt_shape_t& s,
                           const BalanceWorkspace& w, hipStream_t st) {
  balance_kernel<NPL><<<w.groups, 256, 0, st>>>(logits, offsets, s.T, s.N, s.k, w.npad, w.dl, w.part,
                                                reinterpret_cast<uint32_t*>(w.zero_row));
}

BalanceWorkspace plan_balance(const spt_shape_t& s, void* ws) {
  char* p = static_cast<char*>(ws);
  size_t o = 0;
  BalanceWorkspace w = {};
  auto take = [&](size_t bytes) { void* r = p + o; o += align256(bytes); return r; };
  w.npad = (s.N + 31) / 32 * 32;
  w.groups = (s.T + 4 * kBalTokPerWave - 1) / (4 * kBalTokPerWave);
  w.chunk = 512;
  while ((s.T + w.chunk - 1) / w.chunk > 1024) w.chunk *= 2;
  w.nchunks = (s.T + w.chunk - 1) / w.chunk;
  w.dl = static_cast<uint16_t*>(take((size_t)s.T * w.npad * 2));
  w.part = static_cast<float*>(take((size_t)w.groups * 2 * s.N * 4));
  w.gchunks = static_cast<float*>(take((size_t)w.nchunks * w.npad * s.d * 4));
  w.c_off = static_cast<int32_t*>(take((size_t)(w.nchunks + 1) * 4));
  w.c_tok = static_cast<int32_t*>(take((size_t)s.T * 4));
  w.c_border = static_cast<int32_t*>(take((size_t)w.nchunks * 4));
  w.zero_row = static_cast<uint16_t*>(take(256));
  w.bytes = o;
  return w;
}

hipError_t run_router_balance(const spt_shape_t& s, const void* X, const float* logits,
                              const int32_t* offsets, float* loss, float* frac, float* dWr, float* dbr,
                              const BalanceWorkspace& w, hipStream_t st) {
  hipError_t e;
  {
    ScopedKernelTimer tm(kSlotBalance, st);
    const int npl = (s.N + 63) / 64;
    if (npl <= 1) launch_balance<1>(logits, offsets, s, w, st);
    else if (npl <= 2) launch_balance<2>(logits, offsets, s, w, st);
    else if (npl <= 4) launch_balance<4>(logits, offsets, s, w, st);
    else if (npl <= 8) launch_balance<8>(logits, offsets, s, w, st);
    else launch_balance<16>(logits, offsets, s, w, st);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    balance_reduce_kernel<<<1, 1024, 0, st>>>(w.part, offsets, w.groups, s.T, s.N, s.k, loss, frac, dbr);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if ((e = lora_chunks(s.T, w.chunk, w.nchunks, w.c_off, w.c_tok, w.c_border, st)) != hipSuccess) return e;
  }
  // dW_r[i][b] = sum_t X[t][i] dlogit[t][b]: the weight-gradient GEMM over token chunks (the
  // "hidden units" are the blocks), then a fixed-order sum over the chunks
  e = launch_dw(static_cast<const uint16_t*>(X), w.dl, false, w.c_off, w.c_tok, w.c_border, w.zero_row, w.nchunks,
                w.npad, s.d, w.gchunks, kSlotBalance, st);
  if (e != hipSuccess) return e;
  return lora_reduce(w.gchunks, w.nchunks, w.npad, s.d, true, false, dWr, s.d, s.N, st);
}

}  // namespace spt
