// Work list for rows with more than kBigDeg in-neighbours: each such row is cut into chunks of
// kBigChunk neighbours, one workgroup per chunk, then one wave per row combines its chunks in
// order.  The chunk prefix is built on the host from the degrees of the listed rows.
#pragma once
#include <vector>

#include "ctx.h"

namespace ink {

#ifndef INK_BIG_CHUNK
#define INK_BIG_CHUNK 1024
#endif
constexpr int kBigChunk = INK_BIG_CHUNK;
constexpr int kBigSliceChunks = 65536;     // chunks whose partial rows are kept at one time

template <int DUMMY>
__global__ void k_big_degs(const int32_t *list, int n, const int32_t *deg, int32_t *out) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) out[i] = deg[list[i]];
}

struct BigSlice { int row0, row1, chunk0, chunk1; };

// fills c->big_pref (device, n_big + 1 ints) and returns the slices to run
inline hipError_t plan_big_rows(ink_ctx *c, int n_big, const int32_t *in_deg, std::vector<BigSlice> &slices) {
  INK_TRY(c->big_deg.reserve((size_t)n_big * 4));
  INK_TRY(c->big_pref.reserve((size_t)(n_big + 1) * 4));
  hipLaunchKernelGGL((k_big_degs<0>), dim3((n_big + 255) / 256), dim3(256), 0, c->stream,
                     (const int32_t *)c->big_list.as<int32_t>(), n_big, in_deg, c->big_deg.as<int32_t>());
  std::vector<int32_t> deg((size_t)n_big), pref((size_t)n_big + 1);
  INK_TRY(hipMemcpyAsync(deg.data(), c->big_deg.p, (size_t)n_big * 4, hipMemcpyDeviceToHost, c->stream));
  INK_TRY(hipStreamSynchronize(c->stream));
  pref[0] = 0;
  for (int i = 0; i < n_big; i++) pref[i + 1] = pref[i] + (deg[i] + kBigChunk - 1) / kBigChunk;
  INK_TRY(hipMemcpyAsync(c->big_pref.p, pref.data(), pref.size() * 4, hipMemcpyHostToDevice, c->stream));
  INK_TRY(hipStreamSynchronize(c->stream));       // pref is a stack-local vector
  slices.clear();
  int r0 = 0;
  while (r0 < n_big) {
    int r1 = r0 + 1;
    while (r1 < n_big && pref[r1 + 1] - pref[r0] <= kBigSliceChunks) r1++;
    slices.push_back({r0, r1, pref[r0], pref[r1]});
    r0 = r1;
  }
  return hipSuccess;
}

// (row index in the list, first neighbour, end neighbour) of the chunk handled by this workgroup
__device__ __forceinline__ void big_chunk_of_block(const int32_t *pref, int row0, int row1, int chunk0,
                                                   const int32_t *list, const int32_t *in_deg, int &i, int &v,
                                                   int64_t &j0, int64_t &j1) {
  int cg = chunk0 + blockIdx.x;
  int lo = row0, hi = row1 - 1;
  while (lo < hi) {
    int mid = (lo + hi + 1) >> 1;
    if (pref[mid] <= cg) lo = mid; else hi = mid - 1;
  }
  i = lo;
  v = list[i];
  int64_t deg = in_deg[v];
  j0 = (int64_t)(cg - pref[i]) * kBigChunk;
  j1 = j0 + kBigChunk < deg ? j0 + kBigChunk : deg;
}

}  // namespace ink
