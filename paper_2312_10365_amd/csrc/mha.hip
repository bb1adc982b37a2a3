// Sparse multi-head attention of SPT (section 4.1: Eq. 6, Algorithm 1; section 5.1: Algorithms 2
// and 3, CSR with a fixed row length) for gfx950.
//
// None of this is a dense contraction: every step gathers 128/256-byte rows through an index list,
// so the kernels are organised around coalesced row access and the L2 (the K, V, Q, dY rows of one
// sequence are 64-128 KiB and stay cache-resident while its queries run), not around MFMA.
//
//   pq_assign_kernel   one thread per (vector, codebook): fused distance + argmin, codebooks in LDS
//   topl_kernel        one wavefront per query: Eq. 6 scores with byte-compare bit tricks, the
//                      bucket sort of Algorithm 3 as two ballot passes (count, then place)
//   attn_row_kernel    one wavefront per query, used for both directions: lane-per-entry dot
//                      products against gathered rows, wave softmax (forward) or its Jacobian
//                      (backward), then lanes-over-channels accumulation of gathered rows
//   attn_kv_kernel     one wavefront per key: walks the queries that kept the key in ascending
//                      order (bit row + slot bytes written by the backward row kernel) and sums
//                      dK, dV without floating-point atomics
#include <math.h>

#include "../../include/spt_mha.h"
#include "profile.hpp"
#include "spt_device.hpp"
#include "spt_host.hpp"

namespace spt {
namespace {

constexpr int kDp = 8;          // dimensions per codeword (section 5.1)
constexpr int kMaxE = 16;       // codewords per codebook
constexpr int kCbPad = 4;       // floats of padding between codebooks in LDS (bank spread)

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), c, false);
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// ---------------------------------------------------------------- Algorithm 2, lines 2-3
template <int M>
__global__ __launch_bounds__(256) void pq_assign_kernel(const uint16_t* __restrict__ X,
                                                        const float* __restrict__ C,
                                                        uint8_t* __restrict__ codes, int n, int H, int E) {
  constexpr int kStride = kMaxE * kDp + kCbPad;
  __shared__ float cb[M * kStride];
  const int s = blockIdx.y;
  const int head = s % H;
  for (int t = threadIdx.x; t < M * E * kDp; t += 256) {
    const int m = t / (E * kDp), r = t - m * E * kDp;
    cb[m * kStride + r] = C[(size_t)head * M * E * kDp + t];
  }
  __syncthreads();
  const int v0 = blockIdx.x * 256;
  const int nv = min(256, n - v0);
  const size_t base = (size_t)s * n + v0;
  for (int t = threadIdx.x; t < nv * M; t += 256) {
    const int m = t % M;
    const u32x4 raw = *reinterpret_cast<const u32x4*>(X + base * (M * kDp) + (size_t)t * kDp);
    float x[kDp];
#pragma unroll
    for (int w = 0; w < 4; ++w) { x[2 * w] = lo_bf16(raw[w]); x[2 * w + 1] = hi_bf16(raw[w]); }
    const float* c = cb + m * kStride;
    float best = INFINITY;
    int arg = 0;
    for (int e = 0; e < E; ++e) {
      float dist = 0.f;
#pragma unroll
      for (int j = 0; j < kDp; ++j) {
        const float df = x[j] - c[e * kDp + j];
        dist = fmaf(df, df, dist);
      }
      if (dist < best) { best = dist; arg = e; }   // strict: ties stay with the lower index
    }
    codes[base * M + t] = (uint8_t)arg;
  }
}

// ---------------------------------------------------------------- Algorithm 3 with Eq. 6
// Number of equal bytes among the M code bytes of a query and a key.  Per 32-bit word: after the
// XOR a byte is zero exactly where the codes agree; the add cannot carry between bytes because
// bit 7 is masked off first, so the test is exact.
template <int W>
__device__ __forceinline__ int pq_score(const uint32_t (&kc)[W], const uint32_t (&qc)[W]) {
  int sc = 0;
#pragma unroll
  for (int w = 0; w < W; ++w) {
    const uint32_t x = kc[w] ^ qc[w];
    const uint32_t y = ~(((x & 0x7F7F7F7Fu) + 0x7F7F7F7Fu) | x | 0x7F7F7F7Fu);
    sc += __popc(y);
  }
  return sc;
}

// The bucket sort, restated for a wavefront: keys arrive in index order, so bucket s holds the
// keys of score s in index order and only its first L-1 are ever read; the output is those
// prefixes concatenated from score M down, cut at L, padded with -1.  Pass 1 counts each score
// (ballots), pass 2 places every key by its rank inside its score.
template <int M>
__global__ __launch_bounds__(256) void topl_kernel(const uint8_t* __restrict__ cq,
                                                   const uint8_t* __restrict__ ck,
                                                   int32_t* __restrict__ idx, int n, int L, int qpb) {
  constexpr int W = M / 4;
  extern __shared__ uint32_t kcodes[];   // [n][W]
  const int s = blockIdx.y;
  {
    const uint32_t* src = reinterpret_cast<const uint32_t*>(ck + (size_t)s * n * M);
    for (int t = threadIdx.x; t < n * W; t += 256) kcodes[t] = src[t];
  }
  __syncthreads();
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const uint64_t below = (1ull << lane) - 1ull;
  const int q0 = blockIdx.x * qpb;
  const int q1 = min(q0 + qpb, n);
  for (int qi = q0 + wave; qi < q1; qi += 4) {
    uint32_t qc[W];
    {
      const uint32_t* qsrc = reinterpret_cast<const uint32_t*>(cq + ((size_t)s * n + qi) * M);
#pragma unroll
      for (int w = 0; w < W; ++w) qc[w] = __builtin_amdgcn_readfirstlane(qsrc[w]);
    }
    int cnt[M + 1];
#pragma unroll
    for (int b = 0; b <= M; ++b) cnt[b] = 0;
    for (int j0 = 0; j0 < n; j0 += 64) {
      const int j = j0 + lane;
      int sc = -1;
      if (j < n) {
        uint32_t kc[W];
#pragma unroll
        for (int w = 0; w < W; ++w) kc[w] = kcodes[j * W + w];
        sc = pq_score<W>(kc, qc);
      }
#pragma unroll
      for (int b = 0; b <= M; ++b) cnt[b] += __popcll(__ballot(sc == b));
    }
    int base[M + 1];
    int acc = 0;
#pragma unroll
    for (int b = M; b >= 0; --b) { base[b] = acc; acc += min(cnt[b], L - 1); }
    const int total = min(acc, L);
    int32_t* out = idx + ((size_t)s * n + qi) * L;
    int run[M + 1];
#pragma unroll
    for (int b = 0; b <= M; ++b) run[b] = 0;
    for (int j0 = 0; j0 < n; j0 += 64) {
      const int j = j0 + lane;
      int sc = -1;
      if (j < n) {
        uint32_t kc[W];
#pragma unroll
        for (int w = 0; w < W; ++w) kc[w] = kcodes[j * W + w];
        sc = pq_score<W>(kc, qc);
      }
#pragma unroll
      for (int b = 0; b <= M; ++b) {
        if (base[b] < L) {             // uniform: buckets past the cut are never read
          const uint64_t mask = __ballot(sc == b);
          if (sc == b) {
            const int r = run[b] + __popcll(mask & below);
            const int pos = base[b] + r;
            if (r < L - 1 && pos < L) out[pos] = j;
          }
          run[b] += __popcll(mask);
        }
      }
    }
    for (int pos = total + lane; pos < L; pos += 64) out[pos] = -1;
  }
}

// ---------------------------------------------------------------- Algorithm 1, lines 4-5 and their backward
// One wavefront per query row v.  With (R, G1, G2) = (Q, K, V) this is the forward pass:
//   w_l = softmax_l(scale * R[v] . G1[idx_l]),  Out[v] = sum_l w_l G2[idx_l],  A <- w.
// With (R, G1, G2) = (dY, V, K) it is the query side of the backward pass:
//   dA_l = R[v] . G1[idx_l],  w_l = A_l (dA_l - sum_m A_m dA_m) scale,  Out[v] = sum_l w_l G2[idx_l],
// and w is kept (dS) together with, per key, the bit "query i kept me" and the slot it sits in.
// Phase 1 puts entry l on lane l % 64; phase 2 puts 4 channels on each lane, so that DH/4 lanes
// cover a row and 64/(DH/4) entries are in flight per step.
template <int DH, int LPL, bool BWD>
__global__ __launch_bounds__(256) void attn_row_kernel(const uint16_t* __restrict__ R,
                                                       const uint16_t* __restrict__ G1,
                                                       const uint16_t* __restrict__ G2,
                                                       const int32_t* __restrict__ idx,
                                                       float* __restrict__ A, float* __restrict__ dS,
                                                       uint16_t* __restrict__ Out,
                                                       uint32_t* __restrict__ bits,
                                                       uint8_t* __restrict__ slot, int n, int L, float scale) {
  constexpr int NC = DH / 8;           // 16-byte chunks per row
  constexpr int LPR = DH / 4;          // lanes per row in phase 2
  constexpr int G = 64 / LPR;          // entries per phase-2 step
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int i = blockIdx.x * 4 + wave;
  const int s = blockIdx.y;
  if (i >= n) return;                  // whole wavefront; no barrier follows
  const size_t v = (size_t)s * n + i;
  const uint16_t* g1 = G1 + (size_t)s * n * DH;
  const uint16_t* g2 = G2 + (size_t)s * n * DH;

  u32x4 r[NC];
  {
    const u32x4* rp = reinterpret_cast<const u32x4*>(R + v * DH);
#pragma unroll
    for (int c = 0; c < NC; ++c) r[c] = rp[c];
  }
  int32_t jj[LPL];
  float w[LPL];
#pragma unroll
  for (int c = 0; c < LPL; ++c) {
    const int l = c * 64 + lane;
    jj[c] = (l < L) ? idx[v * L + l] : -1;
    if ((uint32_t)jj[c] >= (uint32_t)n) jj[c] = -1;   // -1 = no key; anything out of range is treated alike
    float dot = 0.f;
    if (jj[c] >= 0) {
      const u32x4* kp = reinterpret_cast<const u32x4*>(g1 + (size_t)jj[c] * DH);
      u32x4 kr[NC];
#pragma unroll
      for (int t = 0; t < NC; ++t) kr[t] = kp[t];
#pragma unroll
      for (int t = 0; t < NC; ++t) {
#pragma unroll
        for (int e = 0; e < 4; ++e) dot = dot2(r[t][e], kr[t][e], dot);
      }
    }
    w[c] = dot;
  }
  if (!BWD) {
    float mx = -INFINITY;
#pragma unroll
    for (int c = 0; c < LPL; ++c) {
      w[c] = (jj[c] >= 0) ? w[c] * scale : -INFINITY;
      mx = fmaxf(mx, w[c]);
    }
    mx = wave_max(mx);
    float sum = 0.f;
#pragma unroll
    for (int c = 0; c < LPL; ++c) {
      w[c] = (jj[c] >= 0) ? __expf(w[c] - mx) : 0.f;
      sum += w[c];
    }
    sum = wave_sum(sum);
    const float inv = sum > 0.f ? 1.0f / sum : 0.f;
#pragma unroll
    for (int c = 0; c < LPL; ++c) {
      w[c] *= inv;
      const int l = c * 64 + lane;
      if (l < L) A[v * L + l] = w[c];
    }
  } else {
    float a[LPL];
    float part = 0.f;
#pragma unroll
    for (int c = 0; c < LPL; ++c) {
      const int l = c * 64 + lane;
      a[c] = (jj[c] >= 0) ? A[v * L + l] : 0.f;
      part = fmaf(a[c], w[c], part);
    }
    const float dotsum = wave_sum(part);
    const int nw = (n + 31) >> 5;
#pragma unroll
    for (int c = 0; c < LPL; ++c) {
      const int l = c * 64 + lane;
      w[c] = a[c] * (w[c] - dotsum) * scale;
      if (l < L) dS[v * L + l] = w[c];
      if (jj[c] >= 0) {
        const size_t krow = (size_t)s * n + jj[c];
        atomicOr(bits + krow * nw + (i >> 5), 1u << (i & 31));
        slot[krow * n + i] = (uint8_t)l;
      }
    }
  }
  // Phase 2.
#pragma unroll
  for (int c = 0; c < LPL; ++c) {
    if (jj[c] < 0) { jj[c] = 0; w[c] = 0.f; }
  }
  const int g = lane / LPR, ch = (lane % LPR) * 4;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int c = 0; c < LPL; ++c) {
    if (c * 64 < L) {                  // uniform
#pragma unroll 8
      for (int it = 0; it < 64 / G; ++it) {
        const int src = it * G + g;
        const float we = __shfl(w[c], src);
        const int je = __shfl(jj[c], src);
        const u32x2 row = *reinterpret_cast<const u32x2*>(g2 + (size_t)je * DH + ch);
        acc[0] = fmaf(we, lo_bf16(row[0]), acc[0]);
        acc[1] = fmaf(we, hi_bf16(row[0]), acc[1]);
        acc[2] = fmaf(we, lo_bf16(row[1]), acc[2]);
        acc[3] = fmaf(we, hi_bf16(row[1]), acc[3]);
      }
    }
  }
#pragma unroll
  for (int o = LPR; o < 64; o <<= 1) {
#pragma unroll
    for (int e = 0; e < 4; ++e) acc[e] += __shfl_xor(acc[e], o);
  }
  if (g == 0) {
    u32x2 o2;
    o2[0] = pack_bf16x2(acc[0], acc[1]);
    o2[1] = pack_bf16x2(acc[2], acc[3]);
    *reinterpret_cast<u32x2*>(Out + v * DH + ch) = o2;
  }
}

__global__ __launch_bounds__(256) void fill_zero_kernel(uint32_t* __restrict__ p, size_t count) {
  for (size_t t = (size_t)blockIdx.x * 256 + threadIdx.x; t < count; t += (size_t)gridDim.x * 256) p[t] = 0u;
}

// One wavefront per key j: dV[j] = sum_i A[i][l] dY[i], dK[j] = sum_i dS[i][l] Q[i] over the
// queries i that kept j (slot l), in ascending i.  DH = 128: each lane owns 2 channels of both
// sums.  DH = 64: lanes 0-31 own dV, lanes 32-63 own dK.
template <int DH>
__global__ __launch_bounds__(256) void attn_kv_kernel(const uint16_t* __restrict__ Q,
                                                      const uint16_t* __restrict__ dY,
                                                      const float* __restrict__ A,
                                                      const float* __restrict__ dS,
                                                      const uint32_t* __restrict__ bits,
                                                      const uint8_t* __restrict__ slot,
                                                      uint16_t* __restrict__ dK, uint16_t* __restrict__ dV,
                                                      int n, int L) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int j = blockIdx.x * 4 + wave;
  const int s = blockIdx.y;
  if (j >= n) return;
  const int nw = (n + 31) >> 5;
  const size_t krow = (size_t)s * n + j;
  const uint32_t* brow = bits + krow * nw;
  const uint8_t* srow = slot + krow * n;
  const uint32_t* q32 = reinterpret_cast<const uint32_t*>(Q + (size_t)s * n * DH);
  const uint32_t* y32 = reinterpret_cast<const uint32_t*>(dY + (size_t)s * n * DH);
  constexpr int RW = DH / 2;           // 32-bit words per row
  float av[2] = {0.f, 0.f}, ak[2] = {0.f, 0.f};
  for (int base = 0; base < n; base += 64) {
    const int i = base + lane;
    bool sel = false;
    if (i < n) sel = (brow[i >> 5] >> (i & 31)) & 1u;
    uint64_t mask = __ballot(sel);
    float a = 0.f, ds = 0.f;
    if (sel) {
      const size_t e = ((size_t)s * n + i) * L + srow[i];
      a = A[e];
      ds = dS[e];
    }
    while (mask) {
      int t[4];
      float wa[4], wd[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (mask) {
          t[u] = __ffsll((unsigned long long)mask) - 1;
          mask &= mask - 1;
          wa[u] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(a), t[u]));
          wd[u] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(ds), t[u]));
        } else {
          t[u] = t[0]; wa[u] = 0.f; wd[u] = 0.f;
        }
      }
      uint32_t yv[4], qv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const size_t row = (size_t)(base + t[u]) * RW;
        if (DH == 128) {
          yv[u] = y32[row + lane];
          qv[u] = q32[row + lane];
        } else {
          yv[u] = (lane < 32 ? y32 : q32)[row + (lane & 31)];
        }
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (DH == 128) {
          av[0] = fmaf(wa[u], lo_bf16(yv[u]), av[0]);
          av[1] = fmaf(wa[u], hi_bf16(yv[u]), av[1]);
          ak[0] = fmaf(wd[u], lo_bf16(qv[u]), ak[0]);
          ak[1] = fmaf(wd[u], hi_bf16(qv[u]), ak[1]);
        } else {
          const float wsel = lane < 32 ? wa[u] : wd[u];
          av[0] = fmaf(wsel, lo_bf16(yv[u]), av[0]);
          av[1] = fmaf(wsel, hi_bf16(yv[u]), av[1]);
        }
      }
    }
  }
  if (DH == 128) {
    reinterpret_cast<uint32_t*>(dV + krow * DH)[lane] = pack_bf16x2(av[0], av[1]);
    reinterpret_cast<uint32_t*>(dK + krow * DH)[lane] = pack_bf16x2(ak[0], ak[1]);
  } else {
    uint16_t* dst = lane < 32 ? dV : dK;
    reinterpret_cast<uint32_t*>(dst + krow * DH)[lane & 31] = pack_bf16x2(av[0], av[1]);
  }
}

// ---------------------------------------------------------------- host side
struct MhaWorkspace {
  float* dS;        // [S][n][L]
  uint32_t* bits;   // [S][n][ceil(n/32)]: bit i of row j = query i kept key j
  uint8_t* slot;    // [S][n][n]: slot[j][i] = position of key j in query i's list (where the bit is set)
  size_t bits_words;
  size_t bytes;
};

int check_mha(const spt_mha_shape_t* p) {
  if (!p) return SPT_ERR_ARG;
  if (p->S < 1 || p->H < 1 || p->n < 1 || p->dh < 1 || p->M < 1 || p->E < 1 || p->L < 1) return SPT_ERR_ARG;
  if (p->S % p->H != 0 || p->L > p->n || !isfinite(p->scale)) return SPT_ERR_ARG;
  if (p->dh != 64 && p->dh != 128) return SPT_ERR_UNSUPPORTED;
  if (p->M * kDp != p->dh || p->E > kMaxE || p->L > 256 || p->n > 4096 || p->S > 65535) return SPT_ERR_UNSUPPORTED;
  return SPT_OK;
}

MhaWorkspace plan_mha(const spt_mha_shape_t& s, void* ws) {
  MhaWorkspace w;
  char* p = static_cast<char*>(ws);
  size_t off = 0;
  const size_t rows = (size_t)s.S * s.n;
  w.dS = reinterpret_cast<float*>(p + off);      off += align256(rows * s.L * sizeof(float));
  w.bits_words = rows * ((s.n + 31) / 32);
  w.bits = reinterpret_cast<uint32_t*>(p + off); off += align256(w.bits_words * sizeof(uint32_t));
  w.slot = reinterpret_cast<uint8_t*>(p + off);  off += align256(rows * s.n);
  w.bytes = off;
  return w;
}

bool aligned16(const void* p) { return p && (reinterpret_cast<uintptr_t>(p) & 15) == 0; }
bool aligned4(const void* p) { return p && (reinterpret_cast<uintptr_t>(p) & 3) == 0; }

template <int DH, bool BWD>
void launch_row(const spt_mha_shape_t& s, const uint16_t* R, const uint16_t* G1, const uint16_t* G2,
                const int32_t* idx, float* A, float* dS, uint16_t* Out, uint32_t* bits, uint8_t* slot,
                hipStream_t st) {
  const dim3 grid((s.n + 3) / 4, s.S);
  const int lpl = (s.L + 63) / 64;
#define SPT_ROW(LPL_) \
  hipLaunchKernelGGL((attn_row_kernel<DH, LPL_, BWD>), grid, dim3(256), 0, st, R, G1, G2, idx, A, dS, Out, bits, \
                     slot, s.n, s.L, s.scale)
  switch (lpl) {
    case 1: SPT_ROW(1); break;
    case 2: SPT_ROW(2); break;
    case 3: SPT_ROW(3); break;
    default: SPT_ROW(4); break;
  }
#undef SPT_ROW
}

}  // namespace
}  // namespace spt

using namespace spt;

extern "C" {

size_t spt_mha_workspace_bytes(const spt_mha_shape_t* shape) {
  if (check_mha(shape) != SPT_OK) return 0;
  return plan_mha(*shape, nullptr).bytes;
}

int spt_mha_pq_assign(const spt_mha_shape_t* shape, const void* X, const float* C, uint8_t* codes,
                      void* stream) {
  const int rc = check_mha(shape);
  if (rc != SPT_OK) return rc;
  if (!aligned16(X) || !aligned4(C) || !codes) return SPT_ERR_ARG;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const dim3 grid((shape->n + 255) / 256, shape->S);
  {
    ScopedKernelTimer tm(kSlotMhaPq, st);
    if (shape->M == 8)
      hipLaunchKernelGGL(pq_assign_kernel<8>, grid, dim3(256), 0, st, static_cast<const uint16_t*>(X), C, codes,
                         shape->n, shape->H, shape->E);
    else
      hipLaunchKernelGGL(pq_assign_kernel<16>, grid, dim3(256), 0, st, static_cast<const uint16_t*>(X), C, codes,
                         shape->n, shape->H, shape->E);
  }
  return hipGetLastError() == hipSuccess ? SPT_OK : SPT_ERR_HIP;
}

int spt_mha_topl(const spt_mha_shape_t* shape, const uint8_t* cq, const uint8_t* ck, int32_t* idx,
                 void* stream) {
  const int rc = check_mha(shape);
  if (rc != SPT_OK) return rc;
  if (!aligned4(cq) || !aligned4(ck) || !aligned4(idx)) return SPT_ERR_ARG;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int qpb = 16;
  const dim3 grid((shape->n + qpb - 1) / qpb, shape->S);
  const size_t lds = (size_t)shape->n * shape->M;
  {
    ScopedKernelTimer tm(kSlotMhaTopl, st);
    if (shape->M == 8)
      hipLaunchKernelGGL(topl_kernel<8>, grid, dim3(256), lds, st, cq, ck, idx, shape->n, shape->L, qpb);
    else
      hipLaunchKernelGGL(topl_kernel<16>, grid, dim3(256), lds, st, cq, ck, idx, shape->n, shape->L, qpb);
  }
  return hipGetLastError() == hipSuccess ? SPT_OK : SPT_ERR_HIP;
}

int spt_mha_attn_fwd(const spt_mha_shape_t* shape, const void* Q, const void* K, const void* V,
                     const int32_t* idx, float* A, void* Y, void* stream) {
  const int rc = check_mha(shape);
  if (rc != SPT_OK) return rc;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned4(idx) || !aligned4(A) || !aligned16(Y))
    return SPT_ERR_ARG;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const uint16_t* q = static_cast<const uint16_t*>(Q);
  const uint16_t* k = static_cast<const uint16_t*>(K);
  const uint16_t* v = static_cast<const uint16_t*>(V);
  {
    ScopedKernelTimer tm(kSlotMhaFwd, st);
    if (shape->dh == 64)
      launch_row<64, false>(*shape, q, k, v, idx, A, nullptr, static_cast<uint16_t*>(Y), nullptr, nullptr, st);
    else
      launch_row<128, false>(*shape, q, k, v, idx, A, nullptr, static_cast<uint16_t*>(Y), nullptr, nullptr, st);
  }
  return hipGetLastError() == hipSuccess ? SPT_OK : SPT_ERR_HIP;
}

int spt_mha_attn_bwd(const spt_mha_shape_t* shape, const void* Q, const void* K, const void* V,
                     const void* dY, const int32_t* idx, const float* A, void* dQ, void* dK, void* dV,
                     void* ws, size_t ws_bytes, void* stream) {
  const int rc = check_mha(shape);
  if (rc != SPT_OK) return rc;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(dY) || !aligned4(idx) || !aligned4(A) ||
      !aligned16(dQ) || !aligned16(dK) || !aligned16(dV) || !ws || (reinterpret_cast<uintptr_t>(ws) & 255))
    return SPT_ERR_ARG;
  const MhaWorkspace w = plan_mha(*shape, ws);
  if (ws_bytes < w.bytes) return SPT_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const uint16_t* q = static_cast<const uint16_t*>(Q);
  const uint16_t* k = static_cast<const uint16_t*>(K);
  const uint16_t* v = static_cast<const uint16_t*>(V);
  const uint16_t* dy = static_cast<const uint16_t*>(dY);
  float* Amut = const_cast<float*>(A);   // read-only in the backward instantiation
  {
    ScopedKernelTimer tm(kSlotMhaBwdQ, st);
    const int blocks = (int)((w.bits_words + 255) / 256 < 4096 ? (w.bits_words + 255) / 256 : 4096);
    hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(256), 0, st, w.bits, w.bits_words);
    if (shape->dh == 64)
      launch_row<64, true>(*shape, dy, v, k, idx, Amut, w.dS, static_cast<uint16_t*>(dQ), w.bits, w.slot, st);
    else
      launch_row<128, true>(*shape, dy, v, k, idx, Amut, w.dS, static_cast<uint16_t*>(dQ), w.bits, w.slot, st);
  }
  {
    ScopedKernelTimer tm(kSlotMhaBwdKV, st);
    const dim3 grid((shape->n + 3) / 4, shape->S);
    if (shape->dh == 64)
      hipLaunchKernelGGL(attn_kv_kernel<64>, grid, dim3(256), 0, st, q, dy, A, w.dS, w.bits, w.slot,
                         static_cast<uint16_t*>(dK), static_cast<uint16_t*>(dV), shape->n, shape->L);
    else
      hipLaunchKernelGGL(attn_kv_kernel<128>, grid, dim3(256), 0, st, q, dy, A, w.dS, w.bits, w.slot,
                         static_cast<uint16_t*>(dK), static_cast<uint16_t*>(dV), shape->n, shape->L);
  }
  return hipGetLastError() == hipSuccess ? SPT_OK : SPT_ERR_HIP;
}

}  // extern "C"
