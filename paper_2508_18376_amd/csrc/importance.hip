// Neuron importance profiling and reconstruction order (paper Sec. 4.2 b).
//
// GEMM-1 is run over the calibration tokens with every routed pair kept.  On the matrix-core path
// its epilogue sums the chosen metric over the rows of each tile and this file adds the tiles of an
// expert; on the generic path GEMM-1 stores the metric per (row, neuron) in fp32 and the rows of each
// expert are summed here (one thread per neuron, rows in order).  Both are deterministic.  An
// importance vector is turned into the permutation "neurons by descending importance, equal values
// by ascending id".
#include "common.h"

namespace dsmoe {

template <typename T>
__device__ __forceinline__ float ld_h(const T* p, size_t i);
template <>
__device__ __forceinline__ float ld_h<float>(const float* p, size_t i) { return p[i]; }
template <>
__device__ __forceinline__ float ld_h<uint16_t>(const uint16_t* p, size_t i) { return bf16_to_f32(p[i]); }

// importance[e][q] = sum over the rows of expert e of H[row][q] (the packed weights must have been
// made with the identity permutation, so column q of H is original neuron q)
// unscale: 2^-h_shift for the metrics that contain the up projection (the packed W3 carries 2^h_shift), else 1
template <typename T>
__global__ __launch_bounds__(256) void colsum_kernel(Layout L, const char* ws, float* importance, float unscale) {
  const int e = blockIdx.y;
  const int q = blockIdx.x * 256 + threadIdx.x;
  if (q >= L.F) return;
  const int32_t* exp_nrows = (const int32_t*)(ws + L.o_exp_nrows);
  const int32_t* exp_row0 = (const int32_t*)(ws + L.o_exp_row0);
  const T* H = (const T*)(ws + L.o_H);
  const int n = exp_nrows[e];
  const size_t r0 = (size_t)(exp_row0[e] - L.sh_rows);
  // rows are added in order (deterministic); eight loads are in flight at a time
  float acc = 0.f;
  int r = 0;
  for (; r + 8 <= n; r += 8) {
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = ld_h<T>(H, (r0 + r + u) * L.F + q);
#pragma unroll
    for (int u = 0; u < 8; ++u) acc += v[u];
  }
  for (; r < n; ++r) acc += ld_h<T>(H, (r0 + r) * L.F + q);
  importance[(size_t)e * L.F + q] = acc * unscale;
}

// MFMA path: the GEMM-1 profiling pass has left one row of F column sums per row tile where the layer
// keeps H; importance[e][q] = the sum of the rows of expert e's tiles, in tile order (deterministic).
__global__ __launch_bounds__(256) void colsum_tiles_kernel(Layout L, const char* ws, float* importance, float unscale) {
  const int e = blockIdx.y;
  const int q = blockIdx.x * 256 + threadIdx.x;
  if (q >= L.F) return;
  const int32_t* exp_nrows = (const int32_t*)(ws + L.o_exp_nrows);
  const int32_t* exp_row0 = (const int32_t*)(ws + L.o_exp_row0);
  const float* table = (const float*)(ws + L.o_H);
  const int nt = (exp_nrows[e] + L.BM - 1) / L.BM;
  const size_t t0 = (size_t)((exp_row0[e] - L.sh_rows) / L.BM);
  float acc = 0.f;
  for (int i = 0; i < nt; ++i) acc += table[(t0 + i) * L.F + q];
  importance[(size_t)e * L.F + q] = acc * unscale;
}

hipError_t launch_colsum(const Layout& L, const char* ws, int metric, float* importance, hipStream_t s) {
  dim3 grid((L.F + 255) / 256, L.E_res), block(256);
  const float unscale = metric >= 2 ? ldexpf(1.f, -L.h_shift) : 1.f;
  if (!L.mfma) colsum_kernel<float><<<grid, block, 0, s>>>(L, ws, importance, unscale);  // the generic path keeps H in fp32
  else colsum_tiles_kernel<<<grid, block, 0, s>>>(L, ws, importance, unscale);
  return hipGetLastError();
}

// perm[e][rank(q)] = q with rank(q) = #{q' : imp[q'] > imp[q], or equal and q' < q}.  A NaN importance
// counts as minus infinity (such neurons come last, by id), so the result is a permutation whatever the input.
constexpr int kRankTile = 1024;
__global__ __launch_bounds__(256) void perm_rank_kernel(int F, const float* importance, int32_t* perm) {
  __shared__ float tile[kRankTile];
  const int e = blockIdx.y;
  const float* imp = importance + (size_t)e * F;
  const int q = blockIdx.x * 256 + threadIdx.x;
  auto key = [](float v) { return v != v ? -INFINITY : v; };
  const float mine = q < F ? key(imp[q]) : 0.f;
  int rank = 0;
  for (int base = 0; base < F; base += kRankTile) {
    __syncthreads();
    for (int i = threadIdx.x; i < kRankTile; i += 256) tile[i] = base + i < F ? key(imp[base + i]) : 0.f;
    __syncthreads();
    const int n = min(kRankTile, F - base);
    for (int i = 0; i < n; ++i) {
      const float o = tile[i];
      rank += (o > mine || (o == mine && base + i < q)) ? 1 : 0;
    }
  }
  if (q < F) perm[(size_t)e * F + rank] = q;
}

hipError_t launch_perm_from_importance(const Layout& L, const float* importance, int32_t* perm, hipStream_t s) {
  dim3 grid((L.F + 255) / 256, L.E_res), block(256);
  perm_rank_kernel<<<grid, block, 0, s>>>(L.F, importance, perm);
  return hipGetLastError();
}

}  // namespace dsmoe
