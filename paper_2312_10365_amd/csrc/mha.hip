// Sparse multi-head attention of SPT (section 4.1: Eq. 6, Algorithm 1; section 5.1: Algorithms 2
// and 3, CSR with a fixed row length) for gfx950.
//
// None of this is a dense contraction: every query gathers its own 128/256-byte rows through an
// index list, so the kernels are organised around coalesced rows, LDS residency and the 64-lane
// wavefront, not around MFMA.
//
//   pq_assign_kernel        one thread per (vector, codebook): fused distance + argmin, codebooks in LDS
//   topl_lane_kernel        Algorithm 3 bit-sliced, one LANE per query: inverted code table in LDS,
//                           carry-save score planes for 32 keys at a time, rows staged in LDS
//   topl_kernel             the same selection with one WAVEFRONT per query (ballot ranks), for
//                           shapes whose table and staging do not fit LDS
//   seq_dots_kernel         one workgroup per sequence, gathered tensor resident in LDS: logits +
//                           softmax (forward) or dA + softmax Jacobian (backward)
//   seq_accum_kernel        same residency: weighted sums of gathered rows (Y, dQ through the index
//                           lists; dV, dK through the transposed lists), rows held as fp16
//   transpose_lists_kernel  one workgroup per sequence: the index lists regrouped by key, each
//                           key's entries in ascending query order (bit matrix in LDS, popcount ranks)
//   attn_row_kernel, attn_kv_kernel   the dots + accumulate pair with rows read from L2 (one
//                           wavefront per query / per key), for sequences too large for LDS
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
                                                        uint8_t* __restrict__ codes,
                                                        float* __restrict__ err, int n, int H, int E) {
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
    if (err) err[base * M + t] = sqrtf(best);   // Algorithm 2, lines 4-5: the quantisation error
  }
}

// ---------------------------------------------------------------- Algorithm 3 with Eq. 6
// Codes are below 16 (E <= 16), so the M codes of a vector pack into M/8 words of 4-bit fields.
__device__ __forceinline__ uint32_t pack_nibbles(uint32_t lo4, uint32_t hi4) {
  auto squeeze = [](uint32_t b) {   // bytes b0 b1 b2 b3 -> 16 bits of nibbles
    return (b & 0xFu) | ((b >> 4) & 0xF0u) | ((b >> 8) & 0xF00u) | ((b >> 12) & 0xF000u);
  };
  return squeeze(lo4) | (squeeze(hi4) << 16);
}
// Number of equal 4-bit fields of a query and a key (Eq. 6).  After the XOR a field is zero
// exactly where the codes agree; the add cannot carry between fields because bit 3 of each is
// masked off first, so the test is exact.
template <int W>
__device__ __forceinline__ int pq_score(const uint32_t (&kc)[W], const uint32_t (&qc)[W]) {
  int sc = 0;
#pragma unroll
  for (int w = 0; w < W; ++w) {
    const uint32_t x = kc[w] ^ qc[w];
    const uint32_t y = ~(((x & 0x77777777u) + 0x77777777u) | x | 0x77777777u);
    sc += __popc(y);
  }
  return sc;
}
// Number of set bits of a wavefront mask below the calling lane.
__device__ __forceinline__ int lanes_below(uint64_t mask) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// The bucket sort, restated for a wavefront: keys arrive in index order, so bucket s holds the
// keys of score s in index order and only its first L-1 are ever read; the output is those
// prefixes concatenated from score M down, cut at L, padded with -1.  Pass 1 counts each score
// (ballots), pass 2 places every key by its rank inside its score; buckets that are empty or lie
// past the cut are skipped as a whole (a uniform test), and inside the pass nothing branches.
template <int M>
__global__ __launch_bounds__(256) void topl_kernel(const uint8_t* __restrict__ cq,
                                                   const uint8_t* __restrict__ ck,
                                                   int32_t* __restrict__ idx, int n, int L, int qpb) {
  constexpr int W = M / 8;
  extern __shared__ uint32_t kcodes[];   // [n][W] packed key codes
  const int s = blockIdx.y;
  {
    const u32x2* src = reinterpret_cast<const u32x2*>(ck + (size_t)s * n * M);
    for (int t = threadIdx.x; t < n * W; t += 256) {
      const u32x2 b = src[t];
      kcodes[t] = pack_nibbles(b[0], b[1]);
    }
  }
  __syncthreads();
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int q0 = blockIdx.x * qpb;
  const int q1 = min(q0 + qpb, n);
  for (int qi = q0 + wave; qi < q1; qi += 4) {
    uint32_t qc[W];
    {
      const u32x2* qsrc = reinterpret_cast<const u32x2*>(cq + ((size_t)s * n + qi) * M);
#pragma unroll
      for (int w = 0; w < W; ++w) {
        const u32x2 b = qsrc[w];
        qc[w] = __builtin_amdgcn_readfirstlane(pack_nibbles(b[0], b[1]));
      }
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
      int r = 0, first = L;              // rank inside the bucket, first output slot of the bucket
#pragma unroll
      for (int b = 0; b <= M; ++b) {
        if (base[b] < L && cnt[b] > 0) {   // uniform
          const uint64_t mask = __ballot(sc == b);
          const int rb = run[b] + lanes_below(mask);
          r = (sc == b) ? rb : r;
          first = (sc == b) ? base[b] : first;
          run[b] += __popcll(mask);
        }
      }
      const int pos = first + r;
      if (r < L - 1 && pos < L) out[pos] = j;
    }
    for (int pos = total + lane; pos < L; pos += 64) out[pos] = -1;
  }
}

// Algorithm 3 again, bit-sliced: one LANE per query.  Per sequence an inverted table is built in
// LDS, table[m][e] = the set of keys (a bit mask over key indices) whose code in codebook m is e.
// A query with codes e_1..e_M reads its M masks and adds them bit-plane-wise (a carry-save adder
// tree on 32 keys at a time), which gives the Eq. 6 score of 32 keys in a few dozen bitwise
// operations; "keys of score s" is then an AND of planes.  Pass A counts every score, pass B emits,
// for each score from M down, the set bits in index order at base[s] + rank, stopping at the
// bucket's readable length L-1 and at the row length L.  Rows are staged in LDS as 16-bit key
// indices and written out whole.  Per query this is roughly a sixth of the wavefront-per-query kernel's
// instructions; that kernel remains for shapes whose table and staging do not fit LDS.
__device__ __forceinline__ void full_add(uint32_t a, uint32_t b, uint32_t c, uint32_t& sum, uint32_t& carry) {
  const uint32_t t = a ^ b;
  sum = t ^ c;
  carry = (a & b) | (c & t);
}
__device__ __forceinline__ void half_add(uint32_t a, uint32_t b, uint32_t& sum, uint32_t& carry) {
  sum = a ^ b;
  carry = a & b;
}
// Bit planes p[0..3] of the number of set bits among eight words, bit position by bit position.
__device__ __forceinline__ void count8(const uint32_t* x, uint32_t (&p)[4]) {
  uint32_t s0, c0, s1, c1, s2, c2, c3, t0, d0, d1;
  full_add(x[0], x[1], x[2], s0, c0);
  full_add(x[3], x[4], x[5], s1, c1);
  half_add(x[6], x[7], s2, c2);
  full_add(s0, s1, s2, p[0], c3);
  full_add(c0, c1, c2, t0, d0);
  half_add(t0, c3, p[1], d1);
  half_add(d0, d1, p[2], p[3]);
}
template <int M>
struct ScorePlanes {
  uint32_t hi[4], lo[4], top;    // products of the two high / two low planes; top: score 16 (M = 16)
  __device__ __forceinline__ void build(const uint32_t* x) {
    uint32_t p[4];
    count8(x, p);
    top = 0u;
    if (M == 16) {
      uint32_t q[4], k0, k1, k2, r0, r1, r2, r3;
      count8(x + 8, q);
      half_add(p[0], q[0], r0, k0);
      full_add(p[1], q[1], k0, r1, k1);
      full_add(p[2], q[2], k1, r2, k2);
      full_add(p[3], q[3], k2, r3, top);
      p[0] = r0; p[1] = r1; p[2] = r2; p[3] = r3;
    }
    const uint32_t n0 = ~p[0], n1 = ~p[1], n2 = ~p[2], n3 = ~p[3];
    lo[0] = n1 & n0; lo[1] = n1 & p[0]; lo[2] = p[1] & n0; lo[3] = p[1] & p[0];
    hi[0] = n3 & n2; hi[1] = n3 & p[2]; hi[2] = p[3] & n2; hi[3] = p[3] & p[2];
    if (M == 16) hi[0] &= ~top;      // score 16 has all four low planes clear
  }
  __device__ __forceinline__ uint32_t level(int sc) const {   // sc is a compile-time constant at every use
    return sc == 16 ? top : (hi[sc >> 2] & lo[sc & 3]);
  }
};

template <int M>
__global__ __launch_bounds__(512) void topl_lane_kernel(const uint8_t* __restrict__ cq,
                                                        const uint8_t* __restrict__ ck,
                                                        int32_t* __restrict__ idx, int n, int L) {
  extern __shared__ uint32_t lsm[];
  const int s = blockIdx.y;
  const int nw = (n + 31) >> 5, nwp = nw + 1;       // padded: the 16 masks of a codebook start on different banks
  uint32_t* table = lsm;                            // [M][16][nwp]
  uint16_t* stage = reinterpret_cast<uint16_t*>(lsm + M * 16 * nwp);   // [waves][64][L + 2] key indices, 0xFFFF = none
  const int tid = threadIdx.x, nthreads = blockDim.x;
  for (int t = tid; t < M * 16 * nwp; t += nthreads) table[t] = 0u;
  __syncthreads();
  for (int j = tid; j < n; j += nthreads) {          // one key per thread: its M codes in one load
    uint32_t cw[M / 4];
    const uint32_t* src = reinterpret_cast<const uint32_t*>(ck + ((size_t)s * n + j) * M);
#pragma unroll
    for (int w = 0; w < M / 4; ++w) cw[w] = src[w];
#pragma unroll
    for (int m = 0; m < M; ++m) {
      const uint32_t e = (cw[m >> 2] >> (8 * (m & 3))) & 15u;
      atomicOr(table + (m * 16 + e) * nwp + (j >> 5), 1u << (j & 31));
    }
  }
  const int wave = tid >> 6, lane = tid & 63;
  const int ls = L + 2;                               // row stride in 16-bit units: an odd number of words
  uint16_t* mystage = stage + (size_t)wave * 64 * ls;
  for (int t = lane; t < 64 * ls; t += 64) mystage[t] = 0xFFFFu;
  __syncthreads();

  const int q0 = blockIdx.x * nthreads + wave * 64;   // first query of this wavefront
  const int qi = q0 + lane;
  const bool live = qi < n;
  int off[M];                                         // word offset of this query's mask in every codebook
  {
    const uint8_t* qsrc = cq + ((size_t)s * n + (live ? qi : 0)) * M;
#pragma unroll
    for (int m = 0; m < M; ++m) off[m] = (m * 16 + (qsrc[m] & 15)) * nwp;
  }
  const uint32_t tail = (n & 31) ? ((1u << (n & 31)) - 1u) : 0xFFFFFFFFu;   // real keys of the last word

  int cnt[M + 1];
#pragma unroll
  for (int b = 0; b <= M; ++b) cnt[b] = 0;
  for (int w = 0; w < nw; ++w) {
    uint32_t x[M];
#pragma unroll
    for (int m = 0; m < M; ++m) x[m] = table[off[m] + w];
    ScorePlanes<M> sp;
    sp.build(x);
    const uint32_t valid = (w == nw - 1) ? tail : 0xFFFFFFFFu;
#pragma unroll
    for (int b = 0; b <= M; ++b) cnt[b] += __popc(sp.level(b) & valid);
  }
  int base[M + 1], quota[M + 1];
  int acc = 0;
#pragma unroll
  for (int b = M; b >= 0; --b) {
    base[b] = acc;
    quota[b] = live ? max(0, min(min(cnt[b], L - 1), L - acc)) : 0;   // keys this bucket contributes
    acc += min(cnt[b], L - 1);
  }
  int run[M + 1];
#pragma unroll
  for (int b = 0; b <= M; ++b) run[b] = 0;
  uint16_t* row = mystage + lane * ls;
  bool need[M + 1];                                   // does any query of this wavefront draw on bucket b
#pragma unroll
  for (int b = 0; b <= M; ++b) need[b] = __ballot(quota[b] > 0) != 0ull;
  for (int w = 0; w < nw; ++w) {
    uint32_t x[M];
#pragma unroll
    for (int m = 0; m < M; ++m) x[m] = table[off[m] + w];
    ScorePlanes<M> sp;
    sp.build(x);
    const uint32_t valid = (w == nw - 1) ? tail : 0xFFFFFFFFu;
#pragma unroll
    for (int b = M; b >= 0; --b) {
      if (need[b]) {                                   // uniform
        uint32_t bits = (run[b] < quota[b]) ? (sp.level(b) & valid) : 0u;
        while (bits) {
          const int bit = __ffs(bits) - 1;
          bits &= bits - 1;
          row[base[b] + run[b]] = (uint16_t)(w * 32 + bit);
          ++run[b];
          if (run[b] >= quota[b]) bits = 0u;
        }
      }
    }
  }
  __syncthreads();
  // stage -> idx, whole rows (lanes over positions)
  for (int r = 0; r < 64; ++r) {
    const int q = q0 + r;
    if (q >= n) break;                                 // uniform
    const uint16_t* src = mystage + r * ls;
    int32_t* dst = idx + ((size_t)s * n + q) * L;
    for (int pos = lane; pos < L; pos += 64) {
      const uint32_t key = src[pos];
      dst[pos] = key == 0xFFFFu ? -1 : (int32_t)key;
    }
  }
}

// ---------------------------------------------------------------- Algorithm 1, lines 4-5 and their backward
// Row accesses are cooperative: DH/8 neighbouring lanes read one 128/256-byte row as 16-byte
// pieces, so a wavefront-wide load touches 64/(DH/8) whole cache lines instead of 64 partial ones.
// Workgroup -> (sequence, block of 4 rows).  Consecutive workgroup ids go round-robin over the 8
// XCDs, each with an L2 of its own: sequence s is pinned to XCD s % 8, so that its K, V, Q, dY rows
// and index lists are fetched into one L2 instead of all eight.
__device__ __forceinline__ bool seq_block(int blocks_per_seq, int S, int& s, int& blk) {
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  s = (slot / blocks_per_seq) * 8 + xcd;
  blk = slot % blocks_per_seq;
  return s < S;
}
inline int seq_block_grid(int blocks_per_seq, int S) { return ((S + 7) / 8) * 8 * blocks_per_seq; }

template <int DH>
struct RowMap {
  static constexpr int LPR = DH / 8;     // lanes per row
  static constexpr int G = 64 / LPR;     // rows per wavefront-wide load
};
__device__ __forceinline__ void fma8(float (&acc)[8], float w, const u32x4& row) {
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    acc[2 * e] = fmaf(w, lo_bf16(row[e]), acc[2 * e]);
    acc[2 * e + 1] = fmaf(w, hi_bf16(row[e]), acc[2 * e + 1]);
  }
}

// One wavefront per query row v.  With (R, G1, G2) = (Q, K, V) this is the forward pass:
//   w_l = softmax_l(scale * R[v] . G1[idx_l]),  Out[v] = sum_l w_l G2[idx_l],  A <- w.
// With (R, G1, G2) = (dY, V, K) it is the query side of the backward pass:
//   dA_l = R[v] . G1[idx_l],  w_l = A_l (dA_l - sum_m A_m dA_m) scale,  Out[v] = sum_l w_l G2[idx_l],
// and w is kept (dS) for the key side.  Entry l lives on lane l % 64 for the softmax; for the row
// work lane = (g, c): group g handles entry step * G + g, c is the 16-byte piece of the row.
template <int DH, int LPL, bool BWD>
__global__ __launch_bounds__(256) void attn_row_kernel(const uint16_t* __restrict__ R,
                                                       const uint16_t* __restrict__ G1,
                                                       const uint16_t* __restrict__ G2,
                                                       const int32_t* __restrict__ idx,
                                                       float* __restrict__ A, float* __restrict__ dS,
                                                       uint16_t* __restrict__ Out, int S, int n, int L,
                                                       float scale) {
  constexpr int LPR = RowMap<DH>::LPR, G = RowMap<DH>::G;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  int s, blk;
  if (!seq_block((n + 3) >> 2, S, s, blk)) return;
  const int i = blk * 4 + wave;
  if (i >= n) return;                  // whole wavefront; no barrier follows
  const size_t v = (size_t)s * n + i;
  const int g = lane / LPR, c = lane % LPR;
  const uint16_t* g1 = G1 + (size_t)s * n * DH + c * 8;
  const uint16_t* g2 = G2 + (size_t)s * n * DH + c * 8;
  const u32x4 r = *reinterpret_cast<const u32x4*>(R + v * DH + c * 8);

  int32_t jj[LPL];
  float w[LPL];
#pragma unroll
  for (int cc = 0; cc < LPL; ++cc) {
    const int l = cc * 64 + lane;
    jj[cc] = (l < L) ? idx[v * L + l] : -1;
    if ((uint32_t)jj[cc] >= (uint32_t)n) jj[cc] = -1;   // -1 = no key; anything out of range is treated alike
    w[cc] = 0.f;
    u32x4 kr[LPR];
#pragma unroll
    for (int it = 0; it < LPR; ++it) {
      if (cc * 64 + it * G < L) {      // uniform
        const int je = __shfl(jj[cc], it * G + g);
        kr[it] = *reinterpret_cast<const u32x4*>(g1 + (size_t)max(je, 0) * DH);
      }
    }
#pragma unroll
    for (int it = 0; it < LPR; ++it) {
      if (cc * 64 + it * G < L) {
        float dot = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) dot = dot2(r[e], kr[it][e], dot);
#pragma unroll
        for (int o = 1; o < LPR; o <<= 1) dot += __shfl_xor(dot, o);
        // entry l = it * G + g' sits in group g' = l % G: fetch it from that group's first lane
        const float got = __shfl(dot, (lane % G) * LPR);
        if (lane / G == it) w[cc] = got;
      }
    }
  }
  if (!BWD) {
    float mx = -INFINITY;
#pragma unroll
    for (int cc = 0; cc < LPL; ++cc) {
      w[cc] = (jj[cc] >= 0) ? w[cc] * scale : -INFINITY;
      mx = fmaxf(mx, w[cc]);
    }
    mx = wave_max(mx);
    float sum = 0.f;
#pragma unroll
    for (int cc = 0; cc < LPL; ++cc) {
      w[cc] = (jj[cc] >= 0) ? __expf(w[cc] - mx) : 0.f;
      sum += w[cc];
    }
    sum = wave_sum(sum);
    const float inv = sum > 0.f ? 1.0f / sum : 0.f;
#pragma unroll
    for (int cc = 0; cc < LPL; ++cc) {
      w[cc] *= inv;
      const int l = cc * 64 + lane;
      if (l < L) A[v * L + l] = w[cc];
    }
  } else {
    float a[LPL];
    float part = 0.f;
#pragma unroll
    for (int cc = 0; cc < LPL; ++cc) {
      const int l = cc * 64 + lane;
      a[cc] = (jj[cc] >= 0) ? A[v * L + l] : 0.f;
      part = fmaf(a[cc], w[cc], part);
    }
    const float dotsum = wave_sum(part);
#pragma unroll
    for (int cc = 0; cc < LPL; ++cc) {
      const int l = cc * 64 + lane;
      w[cc] = a[cc] * (w[cc] - dotsum) * scale;
      if (l < L) dS[v * L + l] = w[cc];
    }
  }
  // Weighted sum of the gathered rows.
#pragma unroll
  for (int cc = 0; cc < LPL; ++cc) {
    if (jj[cc] < 0) { jj[cc] = 0; w[cc] = 0.f; }
  }
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int cc = 0; cc < LPL; ++cc) {
#pragma unroll
    for (int i0 = 0; i0 < LPR; i0 += 4) {
      if (cc * 64 + i0 * G < L) {      // uniform; four steps' loads in flight together
        u32x4 row[4];
        float we[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          we[u] = __shfl(w[cc], (i0 + u) * G + g);
          const int je = __shfl(jj[cc], (i0 + u) * G + g);
          row[u] = *reinterpret_cast<const u32x4*>(g2 + (size_t)je * DH);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) fma8(acc, we[u], row[u]);
      }
    }
  }
#pragma unroll
  for (int o = LPR; o < 64; o <<= 1) {
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] += __shfl_xor(acc[e], o);
  }
  if (g == 0) {
    u32x4 o4;
#pragma unroll
    for (int e = 0; e < 4; ++e) o4[e] = pack_bf16x2(acc[2 * e], acc[2 * e + 1]);
    *reinterpret_cast<u32x4*>(Out + v * DH + c * 8) = o4;
  }
}

// The index lists of one sequence, transposed: for every key j the entries (query i, slot l) that
// name it, in ascending i, as tlist[toff[j] .. toff[j+1]) = (i << 8) | l.  One workgroup per
// sequence.  The order comes from a bit matrix (bit i of row j = query i kept key j; OR-ing bits
// is order-independent): the rank of an entry inside its key's list is the number of set bits
// below i.  Fast variant (kLds): matrix, per-word prefix counts and the list under assembly all
// sit in LDS and the list is written out in order; it needs n * L <= 65536 and
// transpose_lds_bytes(n, L) of LDS.  Otherwise the matrix lives in the workspace, ranks are
// counted word by word and every entry goes straight to its place.
constexpr int kTransposeThreads = 1024;
constexpr size_t kLdsLimit = 160 * 1024;
inline size_t transpose_lds_bytes(int n, int L) {
  const size_t nwp = ((n + 31) / 32) | 1;
  return ((size_t)n + 1) * 4 + (size_t)n * nwp * 4 + ((size_t)n * nwp + 1) * 2 + (size_t)n * L * 2;
}
inline bool transpose_fits_lds(int n, int L) {
  return (size_t)n * L <= 65536 && transpose_lds_bytes(n, L) + 1024 <= kLdsLimit;   // + static scratch
}

// Exclusive scan in place over start[0..n] (n <= 4096).  Thread t owns the PER = ceil((n+1)/1024)
// consecutive values from t * PER; wavefront prefix by shuffles, wavefront totals through LDS: two
// barriers in all.  `wtot` is 16 words of LDS scratch.
__device__ __forceinline__ void block_exclusive_scan(int32_t* start, int n, int tid, int32_t* wtot) {
  const int per = (n + kTransposeThreads) / kTransposeThreads;   // ceil((n + 1) / 1024) <= 5
  const int j0 = tid * per;
  int v[5], local = 0;
#pragma unroll
  for (int e = 0; e < 5; ++e) {
    v[e] = (e < per && j0 + e <= n) ? start[j0 + e] : 0;
    local += v[e];
  }
  const int lane = tid & 63, wave = tid >> 6;
  int incl = local;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int up = __shfl_up(incl, o);
    if (lane >= o) incl += up;
  }
  if (lane == 63) wtot[wave] = incl;
  __syncthreads();
  int before = incl - local;
  for (int wv = 0; wv < wave; ++wv) before += wtot[wv];
#pragma unroll
  for (int e = 0; e < 5; ++e) {
    if (e < per && j0 + e <= n) start[j0 + e] = before;
    before += v[e];
  }
  __syncthreads();
}

template <bool kLds>
__global__ __launch_bounds__(kTransposeThreads) void transpose_lists_kernel(const int32_t* __restrict__ idx,
                                                                            int32_t* __restrict__ toff,
                                                                            uint32_t* __restrict__ tlist,
                                                                            uint32_t* __restrict__ gbits, int n,
                                                                            int L) {
  extern __shared__ uint32_t tsm[];
  __shared__ int32_t wtot[16];
  const int s = blockIdx.x;
  const int nw = (n + 31) >> 5;
  const int tid = threadIdx.x;
  int32_t* start = reinterpret_cast<int32_t*>(tsm);            // [n + 1]
  const int32_t* ix = idx + (size_t)s * n * L;
  uint32_t* tl = tlist + (size_t)s * n * L;
  if (kLds) {
    const int nwp = nw | 1;                                                // odd row stride: rows start on different banks
    uint32_t* bits = tsm + (n + 1);                                        // [n][nwp]
    uint16_t* pre = reinterpret_cast<uint16_t*>(bits + n * nwp);           // [n][nwp] set bits in earlier words
    uint16_t* staged = pre + n * nwp + (n & 1);                            // [n * L] entry numbers (kept 4-byte aligned)
    for (int t = tid; t < n * nwp; t += kTransposeThreads) bits[t] = 0u;
    __syncthreads();
    // (eight index loads in flight per thread: one at a time, each would wait out its own latency)
    for (int e0 = tid; e0 < n * L; e0 += 8 * kTransposeThreads) {
      int jv[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int e = e0 + u * kTransposeThreads;
        jv[u] = (e < n * L) ? ix[e] : -1;
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if ((uint32_t)jv[u] < (uint32_t)n) {
          const int i = (e0 + u * kTransposeThreads) / L;
          atomicOr(bits + jv[u] * nwp + (i >> 5), 1u << (i & 31));
        }
      }
    }
    __syncthreads();
    for (int j = tid; j <= n; j += kTransposeThreads) {
      int cnt = 0;
      if (j < n)
        for (int wd = 0; wd < nw; ++wd) {
          pre[j * nwp + wd] = (uint16_t)cnt;
          cnt += __popc(bits[j * nwp + wd]);
        }
      start[j] = cnt;
    }
    __syncthreads();
    block_exclusive_scan(start, n, tid, wtot);
    for (int j = tid; j <= n; j += kTransposeThreads) toff[(size_t)s * (n + 1) + j] = start[j];
    for (int e0 = tid; e0 < n * L; e0 += 8 * kTransposeThreads) {
      int jv[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int e = e0 + u * kTransposeThreads;
        jv[u] = (e < n * L) ? ix[e] : -1;
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int j = jv[u];
        if ((uint32_t)j < (uint32_t)n) {
          const int e = e0 + u * kTransposeThreads;
          const int i = e / L;
          const int wd = j * nwp + (i >> 5);
          const int rank = pre[wd] + __popc(bits[wd] & ((1u << (i & 31)) - 1u));
          staged[start[j] + rank] = (uint16_t)e;
        }
      }
    }
    __syncthreads();
    const int total = start[n];
    for (int t = tid; t < total; t += kTransposeThreads) {
      const int e = staged[t];
      const int i = e / L;
      tl[t] = ((uint32_t)i << 8) | (uint32_t)(e - i * L);
    }
  } else {
    uint32_t* bits = gbits + (size_t)s * n * nw;
    for (int t = tid; t < n * nw; t += kTransposeThreads) bits[t] = 0u;
    __syncthreads();
    for (int e = tid; e < n * L; e += kTransposeThreads) {
      const int j = ix[e];
      if ((uint32_t)j < (uint32_t)n) {
        const int i = e / L;
        atomicOr(bits + (size_t)j * nw + (i >> 5), 1u << (i & 31));
      }
    }
    __syncthreads();
    for (int j = tid; j <= n; j += kTransposeThreads) {
      int cnt = 0;
      if (j < n)
        for (int wd = 0; wd < nw; ++wd) cnt += __popc(bits[(size_t)j * nw + wd]);
      start[j] = cnt;
    }
    __syncthreads();
    block_exclusive_scan(start, n, tid, wtot);
    for (int j = tid; j <= n; j += kTransposeThreads) toff[(size_t)s * (n + 1) + j] = start[j];
    for (int e = tid; e < n * L; e += kTransposeThreads) {
      const int j = ix[e];
      if ((uint32_t)j < (uint32_t)n) {
        const int i = e / L, l = e - i * L;
        const uint32_t* row = bits + (size_t)j * nw;
        int rank = __popc(row[i >> 5] & ((1u << (i & 31)) - 1u));
        for (int wd = 0; wd < (i >> 5); ++wd) rank += __popc(row[wd]);
        tl[start[j] + rank] = ((uint32_t)i << 8) | (uint32_t)l;
      }
    }
  }
}

// One wavefront per key j: dV[j] = sum A[i][l] dY[i], dK[j] = sum dS[i][l] Q[i] over the
// entries of the key's transposed list.  Group g of lanes takes the entries g, g + G, ... in
// order and the groups are added at the end, so the summation order is a fixed function of the
// list (no atomics).
template <int DH>
__global__ __launch_bounds__(256) void attn_kv_kernel(const uint16_t* __restrict__ Q,
                                                      const uint16_t* __restrict__ dY,
                                                      const float* __restrict__ A,
                                                      const float* __restrict__ dS,
                                                      const int32_t* __restrict__ toff,
                                                      const uint32_t* __restrict__ tlist,
                                                      uint16_t* __restrict__ dK, uint16_t* __restrict__ dV,
                                                      int S, int n, int L) {
  constexpr int LPR = RowMap<DH>::LPR, G = RowMap<DH>::G;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  int s, blk;
  if (!seq_block((n + 3) >> 2, S, s, blk)) return;
  const int j = blk * 4 + wave;
  if (j >= n) return;
  const int g = lane / LPR, c = lane % LPR;
  const int beg = toff[(size_t)s * (n + 1) + j], end = toff[(size_t)s * (n + 1) + j + 1];
  const uint32_t* tl = tlist + (size_t)s * n * L;
  const float* As = A + (size_t)s * n * L;
  const float* dSs = dS + (size_t)s * n * L;
  const uint16_t* qs = Q + (size_t)s * n * DH + c * 8;
  const uint16_t* ys = dY + (size_t)s * n * DH + c * 8;
  float av[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  float ak[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int base = beg; base < end; base += 64) {
    const int cnt = min(64, end - base);
    int qi = 0;
    float a = 0.f, ds = 0.f;
    if (lane < cnt) {
      const uint32_t p = tl[base + lane];
      qi = (int)(p >> 8);
      const size_t e = (size_t)qi * L + (p & 255u);
      a = As[e];
      ds = dSs[e];
    }
#pragma unroll
    for (int i0 = 0; i0 < LPR; i0 += 4) {
      if (i0 * G < cnt) {                // uniform; lanes past cnt carry zero weights and query 0
        u32x4 yr[4], qr[4];
        float wa[4], wd[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int src = (i0 + u) * G + g;
          const int qe = __shfl(qi, src);
          wa[u] = __shfl(a, src);
          wd[u] = __shfl(ds, src);
          yr[u] = *reinterpret_cast<const u32x4*>(ys + (size_t)qe * DH);
          qr[u] = *reinterpret_cast<const u32x4*>(qs + (size_t)qe * DH);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          fma8(av, wa[u], yr[u]);
          fma8(ak, wd[u], qr[u]);
        }
      }
    }
  }
#pragma unroll
  for (int o = LPR; o < 64; o <<= 1) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      av[e] += __shfl_xor(av[e], o);
      ak[e] += __shfl_xor(ak[e], o);
    }
  }
  if (g == 0) {
    const size_t krow = (size_t)s * n + j;
    u32x4 ov, ok;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      ov[e] = pack_bf16x2(av[2 * e], av[2 * e + 1]);
      ok[e] = pack_bf16x2(ak[2 * e], ak[2 * e + 1]);
    }
    *reinterpret_cast<u32x4*>(dV + krow * DH + c * 8) = ov;
    *reinterpret_cast<u32x4*>(dK + krow * DH + c * 8) = ok;
  }
}

// ---------------------------------------------------------------- sequence-resident variants
// When one tensor of a sequence fits LDS (n * dh <= 65536 elements) a workgroup of 16 wavefronts
// takes a whole sequence: it copies the rows that will be gathered (K, V, Q or dY of that
// sequence) into LDS once, with a stride of dh*2 + 16 bytes so that rows start on different
// banks, and every gather after that is an LDS read.  The work splits into a "dots" kernel
// (logits / dA, then the softmax or its Jacobian) and an "accumulate" kernel (weighted row sums),
// each with its own tensor resident.
constexpr int kSeqThreads = 1024;
constexpr int kSeqWaves = kSeqThreads / 64;
template <int DH>
struct SeqTile {
  static constexpr int STRIDE = DH * 2 + 16;   // bytes between rows in LDS
};
inline bool seq_resident(int n, int dh) { return (size_t)n * dh <= 65536; }
inline size_t seq_lds_bytes(int n, int dh) { return (size_t)n * (dh * 2 + 16); }

template <int DH>
__device__ __forceinline__ void stage_rows(const uint16_t* __restrict__ src, uint8_t* smem, int n) {
  constexpr int NC = DH / 8;
  const u32x4* g = reinterpret_cast<const u32x4*>(src);
  for (int q0 = threadIdx.x; q0 < n * NC; q0 += 4 * kSeqThreads) {   // four loads in flight per thread
    u32x4 x[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int q = q0 + u * kSeqThreads;
      if (q < n * NC) x[u] = g[q];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int q = q0 + u * kSeqThreads;
      if (q < n * NC) {
        const int row = q / NC, c = q - row * NC;
        *reinterpret_cast<u32x4*>(smem + row * SeqTile<DH>::STRIDE + c * 16) = x[u];
      }
    }
  }
}

// The accumulate kernel multiplies every gathered element once, so the rows are staged as fp16:
// v_fma_mix_f32 then takes them straight from their 16-bit halves, where bf16 would need a shift or
// mask per element first.  The rows are divided by a power of two >= the largest magnitude of the
// sequence beforehand (exact), which puts every value within 2^-14 of that maximum exactly on an
// fp16 number (fp16 has 3 more mantissa bits than bf16) and rounds smaller ones to multiples of
// 2^-24 of the scale: an absolute error below 6e-8 of the largest element.  Returns the scale.
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
template <int DH>
__device__ __forceinline__ float stage_rows_f16(const uint16_t* __restrict__ src, uint8_t* smem, int n,
                                                uint32_t* red /* [kSeqWaves + 1] words of LDS */) {
  constexpr int NC = DH / 8;
  const u32x4* gsrc = reinterpret_cast<const u32x4*>(src);
  uint32_t mag = 0u;                       // largest |x| as a bf16 bit pattern (monotonic in |x|)
  for (int q0 = threadIdx.x; q0 < n * NC; q0 += 4 * kSeqThreads) {   // four loads in flight per thread
    u32x4 xv[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int q = q0 + u * kSeqThreads;
      xv[u] = (q < n * NC) ? gsrc[q] : u32x4{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int q = q0 + u * kSeqThreads;
      if (q < n * NC) {
        const int row = q / NC, c = q - row * NC;
        *reinterpret_cast<u32x4*>(smem + row * SeqTile<DH>::STRIDE + c * 16) = xv[u];
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        mag = max(mag, xv[u][e] & 0x7FFFu);
        mag = max(mag, (xv[u][e] >> 16) & 0x7FFFu);
      }
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mag = max(mag, (uint32_t)__shfl_xor((int)mag, o));
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mag;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t m = 0u;
    for (int wv = 0; wv < kSeqWaves; ++wv) m = max(m, red[wv]);
    red[kSeqWaves] = m;
  }
  __syncthreads();
  const int expo = (int)(red[kSeqWaves] >> 7);          // biased exponent of the largest magnitude
  const float down = expo ? ldexpf(1.0f, 126 - expo) : 1.0f;   // 1 / 2^(expo - 126): |x| * down < 1
  const float up = expo ? ldexpf(1.0f, expo - 126) : 1.0f;
  for (int q = threadIdx.x; q < n * NC; q += kSeqThreads) {
    const int row = q / NC, c = q - row * NC;
    u32x4* slot = reinterpret_cast<u32x4*>(smem + row * SeqTile<DH>::STRIDE + c * 16);
    const u32x4 x = *slot;
    f16x8 h;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      h[2 * e] = (_Float16)(lo_bf16(x[e]) * down);
      h[2 * e + 1] = (_Float16)(hi_bf16(x[e]) * down);
    }
    *slot = __builtin_bit_cast(u32x4, h);
  }
  __syncthreads();
  return up;
}
__device__ __forceinline__ void fma8h(float (&acc)[8], float w, const u32x4& row) {
  const f16x8 h = __builtin_bit_cast(f16x8, row);
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = fmaf((float)h[e], w, acc[e]);
}

// Sum over the DH/8 lanes that share a row, with DPP only (quads, then half rows, then rows).
template <int CTRL>
__device__ __forceinline__ float dpp_move(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, false));
}
template <int LPR>
__device__ __forceinline__ float group_sum(float x) {
  x += dpp_move<0xB1>(x);      // quad_perm [1,0,3,2]
  x += dpp_move<0x4E>(x);      // quad_perm [2,3,0,1]
  x += dpp_move<0x141>(x);     // row_half_mirror: lane k of 8 reads lane 7-k
  if (LPR == 16) x += dpp_move<0x140>(x);   // row_mirror: lane k of 16 reads lane 15-k
  return x;
}
// Whole-wavefront reductions without LDS traffic: DPP inside a row of 16 lanes, then the
// gfx950 row / half swaps (v_permlane16_swap exchanges the odd rows of its first operand with the
// even rows of its second; with the same value in both, first + second is the xor-16 butterfly;
// v_permlane32_swap does the same with the two halves).
struct OpAdd { __device__ static float f(float a, float b) { return a + b; } };
struct OpMax { __device__ static float f(float a, float b) { return fmaxf(a, b); } };
template <class Op>
__device__ __forceinline__ float swap16(float x) {
  const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return Op::f(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
template <class Op>
__device__ __forceinline__ float swap32(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return Op::f(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
template <class Op>
__device__ __forceinline__ float wave_all(float x) {
  x = Op::f(x, dpp_move<0xB1>(x));
  x = Op::f(x, dpp_move<0x4E>(x));
  x = Op::f(x, dpp_move<0x141>(x));
  x = Op::f(x, dpp_move<0x140>(x));
  x = swap16<Op>(x);
  return swap32<Op>(x);
}
// Two values reduced for the price of one: after the row swap, first + second holds the xor-16
// sums of `a` in the even rows and those of `b` in the odd rows (likewise for the halves).
__device__ __forceinline__ float pair16(float a, float b) {
  const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(a), __float_as_uint(b), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float pair32(float a, float b) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(a), __float_as_uint(b), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
// "Dots": G1 rows of the sequence resident.  Forward: A = softmax(scale * R . G1[idx]).  Backward:
// dS = A (dA - sum A dA) scale with dA = R . G1[idx] (R = dY, G1 = V).  Lane (g, c) OWNS entry
// c * G + g of every block of 64 entries (it loads that entry's index and A value and stores its
// result); in step `it` the DH/8 lanes of group g work together on the entry owned by the group's
// lane `it`, and that lane keeps the dot product.  The softmax then needs one exp per lane.
template <int DH, int LPL, bool BWD>
__global__ __launch_bounds__(kSeqThreads) void seq_dots_kernel(const uint16_t* __restrict__ R,
                                                               const uint16_t* __restrict__ G1,
                                                               const int32_t* __restrict__ idx,
                                                               const float* __restrict__ Ain,
                                                               float* __restrict__ Wout, int n, int L,
                                                               float scale) {
  constexpr int LPR = RowMap<DH>::LPR, G = RowMap<DH>::G, STRIDE = SeqTile<DH>::STRIDE;
  extern __shared__ uint8_t seq_smem[];
  const int s = blockIdx.x;
  stage_rows<DH>(G1 + (size_t)s * n * DH, seq_smem, n);
  __syncthreads();
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int g = lane / LPR, c = lane % LPR;
  const int own = c * G + g;             // the entry (inside a block of 64) this lane owns
  const uint32_t mine = c * 16;          // byte offset of this lane's piece inside an LDS row
  // One query ahead: the next query's row piece, index list and A values are requested before the
  // current query's arithmetic, so their latency is hidden behind it.
  u32x4 r_next = {0u, 0u, 0u, 0u};
  int jl_next[LPL];
  float al_next[LPL];
  auto request = [&](int i) {
    const size_t v = (size_t)s * n + i;
    r_next = *reinterpret_cast<const u32x4*>(R + v * DH + c * 8);
#pragma unroll
    for (int cc = 0; cc < LPL; ++cc) {
      const int l = cc * 64 + own;
      jl_next[cc] = (l < L) ? idx[v * L + l] : -1;
      al_next[cc] = 0.f;
      if (BWD) al_next[cc] = (l < L) ? Ain[v * L + l] : 0.f;
    }
  };
  if (wave < n) request(wave);
  for (int i = wave; i < n; i += kSeqWaves) {
    const size_t v = (size_t)s * n + i;
    const u32x4 r = r_next;
    int jl[LPL];
    float al[LPL];
#pragma unroll
    for (int cc = 0; cc < LPL; ++cc) { jl[cc] = jl_next[cc]; al[cc] = al_next[cc]; }
    if (i + kSeqWaves < n) request(i + kSeqWaves);
    float w[LPL];
    bool ok[LPL];
#pragma unroll
    for (int cc = 0; cc < LPL; ++cc) {
      ok[cc] = (uint32_t)jl[cc] < (uint32_t)n;     // -1 = no key; anything out of range alike
      const int jrow = ok[cc] ? jl[cc] : 0;
      w[cc] = 0.f;
      // Four steps under one uniform test: no branch between their shuffles and LDS reads.
#pragma unroll
      for (int i0 = 0; i0 < LPR; i0 += 4) {
        if (cc * 64 + i0 * G < L) {
          u32x4 kr[4];
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int je = __shfl(jrow, g * LPR + i0 + u);
            kr[u] = *reinterpret_cast<const u32x4*>(&seq_smem[mine + __umul24((uint32_t)je, (uint32_t)STRIDE)]);
          }
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            float dot = 0.f;
#pragma unroll
            for (int e = 0; e < 4; ++e) dot = dot2(r[e], kr[u][e], dot);
            dot = group_sum<LPR>(dot);
            w[cc] = (c == i0 + u) ? dot : w[cc];
          }
        }
      }
    }
    if (!BWD) {
      float mx = -INFINITY;
#pragma unroll
      for (int cc = 0; cc < LPL; ++cc) {
        w[cc] = ok[cc] ? w[cc] * scale : -INFINITY;
        mx = fmaxf(mx, w[cc]);
      }
      mx = wave_all<OpMax>(mx);
      float sum = 0.f;
#pragma unroll
      for (int cc = 0; cc < LPL; ++cc) {
        w[cc] = ok[cc] ? __expf(w[cc] - mx) : 0.f;
        sum += w[cc];
      }
      sum = wave_all<OpAdd>(sum);
      const float inv = sum > 0.f ? 1.0f / sum : 0.f;
#pragma unroll
      for (int cc = 0; cc < LPL; ++cc) w[cc] *= inv;
    } else {
      float part = 0.f;
#pragma unroll
      for (int cc = 0; cc < LPL; ++cc) {
        al[cc] = ok[cc] ? al[cc] : 0.f;
        part = fmaf(al[cc], w[cc], part);
      }
      const float dotsum = wave_all<OpAdd>(part);
#pragma unroll
      for (int cc = 0; cc < LPL; ++cc) w[cc] = al[cc] * (w[cc] - dotsum) * scale;
    }
#pragma unroll
    for (int cc = 0; cc < LPL; ++cc) {
      const int l = cc * 64 + own;
      if (l < L) Wout[v * L + l] = w[cc];
    }
  }
}

// "Accumulate": the rows to be summed (G2) resident.  Out[row] = sum over the row's entries of
// weight * G2[column].  kKeys = false: output rows are queries, entries idx[v][0..L) with weights
// W[v][l].  kKeys = true: output rows are keys, entries the key's transposed list, (i << 8) | l,
// with weights W[i][l].
template <int DH, bool kKeys>
__global__ __launch_bounds__(kSeqThreads) void seq_accum_kernel(const uint16_t* __restrict__ G2,
                                                                const int32_t* __restrict__ idx,
                                                                const int32_t* __restrict__ toff,
                                                                const uint32_t* __restrict__ tlist,
                                                                const float* __restrict__ W,
                                                                uint16_t* __restrict__ Out, int n, int L,
                                                                int S, int parts) {
  constexpr int LPR = RowMap<DH>::LPR, G = RowMap<DH>::G, STRIDE = SeqTile<DH>::STRIDE;
  extern __shared__ uint8_t seq_smem[];
  // `parts` workgroups share a sequence's output rows (row = part, part + parts, ... in steps of the
  // wavefronts) and run on one XCD (workgroup id mod 8) side by side.
  const int xcd = blockIdx.x & 7, jj = blockIdx.x >> 3;
  const int part = jj % parts, s = (jj / parts) * 8 + xcd;
  if (s >= S) return;
  const float up = stage_rows_f16<DH>(G2 + (size_t)s * n * DH, seq_smem, n,
                                      reinterpret_cast<uint32_t*>(seq_smem + (size_t)n * STRIDE));
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int g = lane / LPR, c = lane % LPR;
  const uint32_t mine = c * 16;          // byte offset of this lane's piece inside an LDS row
  const float* Ws = W + (size_t)s * n * L;
  auto bounds = [&](int row, int& beg, int& end) {
    if (kKeys) {
      beg = toff[(size_t)s * (n + 1) + row];
      end = toff[(size_t)s * (n + 1) + row + 1];
    } else {
      beg = row * L;
      end = beg + L;
    }
  };
  // Entry `base + lane` of the current list: its column and weight (0, 0 past the end).
  auto fetch = [&](int base, int end, int& col, float& wt) {
    col = 0;
    wt = 0.f;
    if (base + lane < end) {
      if (kKeys) {
        const uint32_t p = tlist[(size_t)s * n * L + base + lane];
        col = (int)(p >> 8);
        wt = Ws[(size_t)col * L + (p & 255u)];
      } else {
        col = idx[(size_t)s * n * L + base + lane];
        wt = Ws[base + lane];
        if ((uint32_t)col >= (uint32_t)n) { col = 0; wt = 0.f; }
      }
    }
  };
  // Rows wave, wave + 16, ...; each row's list in chunks of 64 entries.  The chunk after the
  // current one (of this row or the next) is requested before the current one is consumed.
  int row = part * kSeqWaves + wave, beg = 0, end = 0;
  if (row < n) bounds(row, beg, end);
  int base = beg, pcol;
  float pwt;
  fetch(base, end, pcol, pwt);
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  while (row < n) {
    const int col = pcol;
    const float wt = pwt;
    const int cnt = min(64, end - base);
    const bool last = base + 64 >= end;
    int nrow = row, nbase = base + 64, nbeg = beg, nend = end;
    if (last) {
      nrow = row + kSeqWaves * parts;
      nbeg = nend = 0;
      if (nrow < n) bounds(nrow, nbeg, nend);
      nbase = nbeg;
    }
    fetch(nbase, nend, pcol, pwt);
    // A few steps at a time under one uniform test: inside a group nothing branches, so the
    // shuffles and the LDS reads are all in flight before the first multiply.  Lanes past cnt carry
    // weight 0 and column 0.  Index lists are full chunks (groups of 4); the key side's lists end
    // anywhere, so it tests every 2 steps and wastes less on the tail.
    constexpr int GS = kKeys ? 2 : 4;
#pragma unroll
    for (int i0 = 0; i0 < LPR; i0 += GS) {
      if (i0 * G < cnt) {
        u32x4 rowv[GS];
        float we[GS];
#pragma unroll
        for (int u = 0; u < GS; ++u) {
          const int ce = __shfl(col, (i0 + u) * G + g);
          we[u] = __shfl(wt, (i0 + u) * G + g);
          rowv[u] = *reinterpret_cast<const u32x4*>(&seq_smem[mine + __umul24((uint32_t)ce, (uint32_t)STRIDE)]);
        }
#pragma unroll
        for (int u = 0; u < GS; ++u) fma8h(acc, we[u], rowv[u]);
      }
    }
    if (last) {
      // Sum the 8 accumulators over the groups, reduce-scatter fashion: row r (16 lanes) ends up
      // with the totals of channels 2r and 2r + 1 of its lanes' pieces.
      float even = pair32(pair16(acc[0], acc[2]), pair16(acc[4], acc[6]));
      float odd = pair32(pair16(acc[1], acc[3]), pair16(acc[5], acc[7]));
      if (LPR == 8) {                      // two groups share a row: add the other one (lane ^ 8)
        even += dpp_move<0x128>(even);
        odd += dpp_move<0x128>(odd);
      }
      const int r = lane >> 4, pc = lane & 15;
      if (pc < LPR)
        *reinterpret_cast<uint32_t*>(Out + ((size_t)s * n + row) * DH + pc * 8 + 2 * r) =
            pack_bf16x2(even * up, odd * up);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    }
    row = nrow; base = nbase; beg = nbeg; end = nend;
  }
}

// ---------------------------------------------------------------- host side
struct MhaWorkspace {
  float* dS;          // [S][n][L]
  int32_t* toff;      // [S][n + 1]
  uint32_t* tlist;    // [S][n * L]
  uint32_t* gbits;    // [S][n][ceil(n/32)] when the transposition does not fit LDS, else null
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
  w.dS = reinterpret_cast<float*>(p + off);        off += align256(rows * s.L * sizeof(float));
  w.toff = reinterpret_cast<int32_t*>(p + off);    off += align256((size_t)s.S * (s.n + 1) * sizeof(int32_t));
  w.tlist = reinterpret_cast<uint32_t*>(p + off);  off += align256(rows * s.L * sizeof(uint32_t));
  w.gbits = nullptr;
  if (!transpose_fits_lds(s.n, s.L)) {
    w.gbits = reinterpret_cast<uint32_t*>(p + off);
    off += align256(rows * ((s.n + 31) / 32) * sizeof(uint32_t));
  }
  w.bytes = off;
  return w;
}

bool aligned16(const void* p) { return p && (reinterpret_cast<uintptr_t>(p) & 15) == 0; }
bool aligned4(const void* p) { return p && (reinterpret_cast<uintptr_t>(p) & 3) == 0; }

template <int DH, bool BWD>
void launch_row(const spt_mha_shape_t& s, const uint16_t* R, const uint16_t* G1, const uint16_t* G2,
                const int32_t* idx, float* A, float* dS, uint16_t* Out, hipStream_t st) {
  const dim3 grid(seq_block_grid((s.n + 3) / 4, s.S));
  const int lpl = (s.L + 63) / 64;
#define SPT_ROW(LPL_) \
  hipLaunchKernelGGL((attn_row_kernel<DH, LPL_, BWD>), grid, dim3(256), 0, st, R, G1, G2, idx, A, dS, Out, s.S, \
                     s.n, s.L, s.scale)
  switch (lpl) {
    case 1: SPT_ROW(1); break;
    case 2: SPT_ROW(2); break;
    case 3: SPT_ROW(3); break;
    default: SPT_ROW(4); break;
  }
#undef SPT_ROW
}

template <int DH, bool BWD>
void launch_seq_dots(const spt_mha_shape_t& s, const uint16_t* R, const uint16_t* G1, const int32_t* idx,
                     const float* Ain, float* Wout, hipStream_t st) {
  const size_t lds = seq_lds_bytes(s.n, DH);
  const int lpl = (s.L + 63) / 64;
#define SPT_DOTS(LPL_)                                                                                      \
  do {                                                                                                      \
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(seq_dots_kernel<DH, LPL_, BWD>),                \
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);                        \
    hipLaunchKernelGGL((seq_dots_kernel<DH, LPL_, BWD>), dim3(s.S), dim3(kSeqThreads), lds, st, R, G1, idx, \
                       Ain, Wout, s.n, s.L, s.scale);                                                       \
  } while (0)
  switch (lpl) {
    case 1: SPT_DOTS(1); break;
    case 2: SPT_DOTS(2); break;
    case 3: SPT_DOTS(3); break;
    default: SPT_DOTS(4); break;
  }
#undef SPT_DOTS
}

template <int DH, bool kKeys>
void launch_seq_accum(const spt_mha_shape_t& s, const uint16_t* G2, const int32_t* idx, const int32_t* toff,
                      const uint32_t* tlist, const float* W, uint16_t* Out, hipStream_t st) {
  const size_t lds = seq_lds_bytes(s.n, DH) + (kSeqWaves + 1) * sizeof(uint32_t);
  (void)hipFuncSetAttribute(reinterpret_cast<const void*>(seq_accum_kernel<DH, kKeys>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  // Key side, 64-wide heads: two workgroups per sequence.  The weights W[i][l] are gathered 4 bytes at
  // a time out of 2 x 128 KiB per sequence; with 32 sequences resident per XCD that is twice its L2,
  // with 16 it fits (measured 0.285 -> 0.262 ms on the OPT-2048 shape; four parts, or two with
  // 128-wide heads, whose rows take twice as long to stage, cost more than they save).
  const int parts = (kKeys && DH == 64 && s.n >= 2 * kSeqWaves) ? 2 : 1;
  hipLaunchKernelGGL((seq_accum_kernel<DH, kKeys>), dim3(8 * parts * ((s.S + 7) / 8)), dim3(kSeqThreads), lds, st,
                     G2, idx, toff, tlist, W, Out, s.n, s.L, s.S, parts);
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
                      float* err, void* stream) {
  const int rc = check_mha(shape);
  if (rc != SPT_OK) return rc;
  if (!aligned16(X) || !aligned4(C) || !codes || (err && !aligned4(err))) return SPT_ERR_ARG;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const dim3 grid((shape->n + 255) / 256, shape->S);
  {
    ScopedKernelTimer tm(kSlotMhaPq, st);
    if (shape->M == 8)
      hipLaunchKernelGGL(pq_assign_kernel<8>, grid, dim3(256), 0, st, static_cast<const uint16_t*>(X), C, codes,
                         err, shape->n, shape->H, shape->E);
    else
      hipLaunchKernelGGL(pq_assign_kernel<16>, grid, dim3(256), 0, st, static_cast<const uint16_t*>(X), C, codes,
                         err, shape->n, shape->H, shape->E);
  }
  return hipGetLastError() == hipSuccess ? SPT_OK : SPT_ERR_HIP;
}

int spt_mha_topl(const spt_mha_shape_t* shape, const uint8_t* cq, const uint8_t* ck, int32_t* idx,
                 void* stream) {
  const int rc = check_mha(shape);
  if (rc != SPT_OK) return rc;
  if (!cq || !ck || ((reinterpret_cast<uintptr_t>(cq) | reinterpret_cast<uintptr_t>(ck)) & 7) || !aligned4(idx))
    return SPT_ERR_ARG;
  hipStream_t st = static_cast<hipStream_t>(stream);
  ScopedKernelTimer tm(kSlotMhaTopl, st);
  // One lane per query when the inverted table and the row staging fit LDS (up to 8 wavefronts per
  // workgroup share a table; as many as still let two workgroups share a CU); otherwise one
  // wavefront per query.
  const size_t table_bytes = (size_t)shape->M * 16 * ((shape->n + 31) / 32 + 1) * sizeof(uint32_t);
  const size_t stage_bytes = (size_t)64 * (shape->L + 2) * sizeof(uint16_t);
  int waves = 0;
  for (int cand = 8; cand >= 1 && !waves; cand >>= 1)
    if (2 * (table_bytes + cand * stage_bytes) <= kLdsLimit || cand == 1)
      if (table_bytes + cand * stage_bytes <= kLdsLimit) waves = cand;
  if (waves) {
    while (waves > 1 && (waves / 2) * 64 >= shape->n) waves >>= 1;   // short sequences: no idle wavefronts
    const size_t lds = table_bytes + waves * stage_bytes;
    const dim3 grid((shape->n + waves * 64 - 1) / (waves * 64), shape->S);
    if (shape->M == 8) {
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(topl_lane_kernel<8>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      hipLaunchKernelGGL(topl_lane_kernel<8>, grid, dim3(waves * 64), lds, st, cq, ck, idx, shape->n, shape->L);
    } else {
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(topl_lane_kernel<16>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      hipLaunchKernelGGL(topl_lane_kernel<16>, grid, dim3(waves * 64), lds, st, cq, ck, idx, shape->n, shape->L);
    }
  } else {
    const int qpb = 16;
    const dim3 grid((shape->n + qpb - 1) / qpb, shape->S);
    const size_t lds = (size_t)shape->n * (shape->M / 8) * sizeof(uint32_t);
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
    uint16_t* y = static_cast<uint16_t*>(Y);
    if (seq_resident(shape->n, shape->dh)) {
      if (shape->dh == 64) {
        launch_seq_dots<64, false>(*shape, q, k, idx, nullptr, A, st);
        launch_seq_accum<64, false>(*shape, v, idx, nullptr, nullptr, A, y, st);
      } else {
        launch_seq_dots<128, false>(*shape, q, k, idx, nullptr, A, st);
        launch_seq_accum<128, false>(*shape, v, idx, nullptr, nullptr, A, y, st);
      }
    } else if (shape->dh == 64) {
      launch_row<64, false>(*shape, q, k, v, idx, A, nullptr, y, st);
    } else {
      launch_row<128, false>(*shape, q, k, v, idx, A, nullptr, y, st);
    }
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
  const bool resident = seq_resident(shape->n, shape->dh);
  {
    ScopedKernelTimer tm(kSlotMhaBwdQ, st);
    uint16_t* dq = static_cast<uint16_t*>(dQ);
    if (resident) {
      if (shape->dh == 64) {
        launch_seq_dots<64, true>(*shape, dy, v, idx, A, w.dS, st);
        launch_seq_accum<64, false>(*shape, k, idx, nullptr, nullptr, w.dS, dq, st);
      } else {
        launch_seq_dots<128, true>(*shape, dy, v, idx, A, w.dS, st);
        launch_seq_accum<128, false>(*shape, k, idx, nullptr, nullptr, w.dS, dq, st);
      }
    } else if (shape->dh == 64) {
      launch_row<64, true>(*shape, dy, v, k, idx, Amut, w.dS, dq, st);
    } else {
      launch_row<128, true>(*shape, dy, v, k, idx, Amut, w.dS, dq, st);
    }
  }
  {
    ScopedKernelTimer tm(kSlotMhaTranspose, st);
    if (!w.gbits) {
      const size_t lds = transpose_lds_bytes(shape->n, shape->L);
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(transpose_lists_kernel<true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      hipLaunchKernelGGL(transpose_lists_kernel<true>, dim3(shape->S), dim3(kTransposeThreads), lds, st, idx,
                         w.toff, w.tlist, nullptr, shape->n, shape->L);
    } else {
      const size_t lds = ((size_t)shape->n + 1) * sizeof(int32_t);
      hipLaunchKernelGGL(transpose_lists_kernel<false>, dim3(shape->S), dim3(kTransposeThreads), lds, st, idx,
                         w.toff, w.tlist, w.gbits, shape->n, shape->L);
    }
  }
  {
    ScopedKernelTimer tm(kSlotMhaBwdKV, st);
    const dim3 grid(seq_block_grid((shape->n + 3) / 4, shape->S));
    uint16_t* dk = static_cast<uint16_t*>(dK);
    uint16_t* dv = static_cast<uint16_t*>(dV);
    if (resident) {
      if (shape->dh == 64) {
        launch_seq_accum<64, true>(*shape, dy, nullptr, w.toff, w.tlist, A, dv, st);
        launch_seq_accum<64, true>(*shape, q, nullptr, w.toff, w.tlist, w.dS, dk, st);
      } else {
        launch_seq_accum<128, true>(*shape, dy, nullptr, w.toff, w.tlist, A, dv, st);
        launch_seq_accum<128, true>(*shape, q, nullptr, w.toff, w.tlist, w.dS, dk, st);
      }
    } else if (shape->dh == 64)
      hipLaunchKernelGGL(attn_kv_kernel<64>, grid, dim3(256), 0, st, q, dy, A, w.dS, w.toff, w.tlist,
                         static_cast<uint16_t*>(dK), static_cast<uint16_t*>(dV), shape->S, shape->n, shape->L);
    else
      hipLaunchKernelGGL(attn_kv_kernel<128>, grid, dim3(256), 0, st, q, dy, A, w.dS, w.toff, w.tlist,
                         static_cast<uint16_t*>(dK), static_cast<uint16_t*>(dV), shape->S, shape->n, shape->L);
  }
  return hipGetLastError() == hipSuccess ? SPT_OK : SPT_ERR_HIP;
}

}  // extern "C"
