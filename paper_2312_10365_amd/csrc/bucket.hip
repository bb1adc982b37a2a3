// Token batching by activated block: Algorithm 4's per-block token selection, done once
// for all blocks as a stable counting sort of the (token, slot) pairs by block id.
//
// Three small integer kernels, exact and deterministic:
//   1. per chunk of 128 tokens, a (block x token) membership bitmask in LDS gives the
//      chunk's histogram;
//   2. one workgroup turns the chunk histograms into bucket offsets and per-chunk bases;
//   3. each chunk rebuilds its bitmask; the rank of a pair inside its bucket is the chunk
//      base plus the number of lower tokens of the chunk in the same bucket (popcount).
// A token lists each block at most once, so one bit per (block, token) is enough, and the
// order inside a bucket is by token id, i.e. stable.
#include "spt_device.hpp"
#include "spt_host.hpp"
#include "profile.hpp"

namespace spt {

constexpr int kWordsPerChunk = kBucketChunkTokens / 32;

__device__ __forceinline__ void build_chunk_mask(const int32_t* __restrict__ idx, int T, int N,
                                                 int k, int chunk, uint32_t* mask) {
  for (int e = threadIdx.x; e < N * kWordsPerChunk; e += blockDim.x) mask[e] = 0u;
  __syncthreads();
  const int t0 = chunk * kBucketChunkTokens;
  const int nt = min(kBucketChunkTokens, T - t0);
  const int64_t p0 = (int64_t)t0 * k;
  // (eight loads in flight per thread: one at a time, each waits out its own latency)
  for (int e0 = threadIdx.x; e0 < nt * k; e0 += 8 * blockDim.x) {
    int bv[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int e = e0 + u * blockDim.x;
      bv[u] = (e < nt * k) ? idx[p0 + e] : -1;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int tl = (e0 + u * blockDim.x) / k;
      if (bv[u] >= 0 && bv[u] < N) atomicOr(&mask[bv[u] * kWordsPerChunk + (tl >> 5)], 1u << (tl & 31));
    }
  }
  __syncthreads();
}

__global__ __launch_bounds__(256) void bucket_hist_kernel(const int32_t* __restrict__ idx, int T,
                                                          int N, int k,
                                                          int32_t* __restrict__ chunk_hist) {
  extern __shared__ uint32_t mask[];
  build_chunk_mask(idx, T, N, k, blockIdx.x, mask);
  for (int b = threadIdx.x; b < N; b += blockDim.x) {
    int c = 0;
#pragma unroll
    for (int w = 0; w < kWordsPerChunk; ++w) c += __popc(mask[b * kWordsPerChunk + w]);
    chunk_hist[(size_t)blockIdx.x * N + b] = c;
  }
}

// One workgroup of 1024 threads; thread b owns bucket b.
__global__ __launch_bounds__(1024) void bucket_scan_kernel(int32_t* __restrict__ chunk_hist,
                                                           int nchunks, int N,
                                                           int32_t* __restrict__ offsets) {
  __shared__ int32_t scan[16];
  const int b = threadIdx.x;
  int total = 0;
  if (b < N) {
    for (int c0 = 0; c0 < nchunks; c0 += 16) {   // sixteen loads in flight, then the running sums
      int v[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) v[u] = (c0 + u < nchunks) ? chunk_hist[(size_t)(c0 + u) * N + b] : 0;
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        if (c0 + u < nchunks) chunk_hist[(size_t)(c0 + u) * N + b] = total;  // pairs of this bucket in earlier chunks
        total += v[u];
      }
    }
  }
  // exclusive scan of the bucket totals: wavefront prefix by shuffles, wavefront sums through LDS
  const int lane = b & 63, wave = b >> 6;
  int incl = total;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int up = __shfl_up(incl, o);
    if (lane >= o) incl += up;
  }
  if (lane == 63) scan[wave] = incl;
  __syncthreads();
  int before = incl - total;
  for (int wv = 0; wv < wave; ++wv) before += scan[wv];
  if (b < N) offsets[b] = before;
  if (b == N - 1) offsets[N] = before + total;
}

__global__ __launch_bounds__(256) void bucket_scatter_kernel(
    const int32_t* __restrict__ idx, int T, int N, int k, const int32_t* __restrict__ chunk_hist,
    const int32_t* __restrict__ offsets, int32_t* __restrict__ perm, int32_t* __restrict__ inv) {
  extern __shared__ uint32_t mask[];
  build_chunk_mask(idx, T, N, k, blockIdx.x, mask);
  const int t0 = blockIdx.x * kBucketChunkTokens;
  const int nt = min(kBucketChunkTokens, T - t0);
  const int64_t p0 = (int64_t)t0 * k;
  for (int e0 = threadIdx.x; e0 < nt * k; e0 += 4 * blockDim.x) {   // four pairs at a time per thread
    int bv[4], base[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int e = e0 + u * blockDim.x;
      bv[u] = (e < nt * k) ? idx[p0 + e] : -1;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const bool ok = bv[u] >= 0 && bv[u] < N;
      base[u] = ok ? offsets[bv[u]] + chunk_hist[(size_t)blockIdx.x * N + bv[u]] : 0;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int e = e0 + u * blockDim.x, b = bv[u];
      if (b < 0 || b >= N) continue;
      const int tl = e / k;
      const uint32_t* m = mask + b * kWordsPerChunk;
      int r = __popc(m[tl >> 5] & ((1u << (tl & 31)) - 1u));
      for (int w = 0; w < (tl >> 5); ++w) r += __popc(m[w]);
      const int q = base[u] + r;
      perm[q] = (int32_t)(p0 + e);
      inv[p0 + e] = q;
    }
  }
}

// Fixed scratch of the allocation-free entry point (spt_bucket_tokens_noalloc): the per-chunk
// histogram table of the three kernels above.  The array's name is only a host-side handle;
// its device address is looked up once per device and used everywhere the memory is meant.
static __device__ __align__(256) int32_t scratch[kStaticBucketScratchInts];

hipError_t bucket_static_scratch(int32_t** out) {
  constexpr int kMaxDevices = 64;
  static int32_t* ptr_of_device[kMaxDevices] = {};
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  if (!ptr_of_device[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));   // the current device's copy of the array
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    ptr_of_device[dev] = static_cast<int32_t*>(p);
  }
  *out = ptr_of_device[dev];
  return hipSuccess;
}

hipError_t run_bucket(const spt_shape_t& s, const int32_t* idx, int32_t* offsets, int32_t* perm,
                      int32_t* inv, int32_t* chunk_hist, hipStream_t st) {
  const int nchunks = (s.T + kBucketChunkTokens - 1) / kBucketChunkTokens;
  const size_t smem = (size_t)s.N * kWordsPerChunk * sizeof(uint32_t);
  {
    ScopedKernelTimer tm(kSlotBucketHist, st);
    bucket_hist_kernel<<<nchunks, 256, smem, st>>>(idx, s.T, s.N, s.k, chunk_hist);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  {
    ScopedKernelTimer tm(kSlotBucketScan, st);
    bucket_scan_kernel<<<1, 1024, 0, st>>>(chunk_hist, nchunks, s.N, offsets);
  }
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  {
    ScopedKernelTimer tm(kSlotBucketScatter, st);
    bucket_scatter_kernel<<<nchunks, 256, smem, st>>>(idx, s.T, s.N, s.k, chunk_hist, offsets, perm,
                                                      inv);
  }
  return hipGetLastError();
}

}  // namespace spt
