// Complete transformation of a layer into E*P finer-grained experts (Sec. 3.1 of the paper, steps
// 1-3): router columns repeated P times, the neurons of every expert (in the order of the static
// permutation of Sec. 4.2 b) split evenly over P new experts, down projections multiplied by P.
// The outputs are plain tensors in the same orientation as the inputs: a layer any MoE
// implementation can run with Top-(K*P).  Pure data movement, one pass over the weights.
#include "common.h"

namespace dsmoe {

template <typename T>
__device__ __forceinline__ T times_p(T v, int P) {
  if constexpr (sizeof(T) == 2) return f32_to_bf16(bf16_to_f32(v) * (float)P);  // product exact in fp32, one rounding to bf16
  else return v * (float)P;
}

// out[e*P+p][d][j] = in[e][d][perm[e][p*Fp + j]]: one workgroup per (e, d) row, neurons across threads
template <typename T>
__global__ __launch_bounds__(256) void transform_w13_kernel(const T* __restrict__ w1, const T* __restrict__ w3,
                                                            const int32_t* __restrict__ perm, T* __restrict__ o1,
                                                            T* __restrict__ o3, int D, int F, int P) {
  const int e = blockIdx.y, d = blockIdx.x, Fp = F / P;
  const T* r1 = w1 + ((size_t)e * D + d) * F;
  const T* r3 = w3 + ((size_t)e * D + d) * F;
  for (int pos = threadIdx.x; pos < F; pos += 256) {
    const int src = perm ? perm[(size_t)e * F + pos] : pos;
    const int p = pos / Fp, j = pos - p * Fp;
    const size_t o = (((size_t)e * P + p) * D + d) * Fp + j;
    o1[o] = r1[src];
    o3[o] = r3[src];
  }
}

// Same mapping for rows that fit in LDS and whose parts are whole 16-byte groups: the two rows are
// read with 16-byte loads into LDS, gathered there, and written with 16-byte stores.
template <typename T>
__global__ __launch_bounds__(256) void transform_w13_lds_kernel(const T* __restrict__ w1, const T* __restrict__ w3,
                                                                const int32_t* __restrict__ perm, T* __restrict__ o1,
                                                                T* __restrict__ o3, int D, int F, int P) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  constexpr int V = 16 / sizeof(T);  // values per 16-byte group
  T* s1 = (T*)smem;
  T* s3 = s1 + F;
  const int e = blockIdx.y, d = blockIdx.x, Fp = F / P;
  const uint4* r1 = (const uint4*)(w1 + ((size_t)e * D + d) * F);
  const uint4* r3 = (const uint4*)(w3 + ((size_t)e * D + d) * F);
  for (int g = threadIdx.x; g < F / V; g += 256) {
    ((uint4*)s1)[g] = r1[g];
    ((uint4*)s3)[g] = r3[g];
  }
  __syncthreads();
  for (int g = threadIdx.x; g < F / V; g += 256) {
    const int pos0 = g * V;
    const int p = pos0 / Fp, j = pos0 - p * Fp;
    T a[V], b[V];
#pragma unroll
    for (int i = 0; i < V; ++i) {
      const int src = perm ? perm[(size_t)e * F + pos0 + i] : pos0 + i;
      a[i] = s1[src];
      b[i] = s3[src];
    }
    const size_t o = (((size_t)e * P + p) * D + d) * Fp + j;
    *(uint4*)(o1 + o) = *(const uint4*)a;
    *(uint4*)(o3 + o) = *(const uint4*)b;
  }
}

// out[e][pos][:] = P * in[e][perm[e][pos]][:] (the [E*P][Fp][D] tensor is the [E][F][D] one with rows reordered)
template <typename T, bool VEC>
__global__ __launch_bounds__(256) void transform_w2_kernel(const T* __restrict__ w2, const int32_t* __restrict__ perm,
                                                           T* __restrict__ o2, int D, int F, int P) {
  const int e = blockIdx.y, pos = blockIdx.x;
  const int src = perm ? perm[(size_t)e * F + pos] : pos;
  const T* in = w2 + ((size_t)e * F + src) * D;
  T* out = o2 + ((size_t)e * F + pos) * D;
  if constexpr (VEC) {  // rows are whole 16-byte groups
    constexpr int V = 16 / sizeof(T);
    for (int g = threadIdx.x; g < D / V; g += 256) {
      uint4 raw = ((const uint4*)in)[g];
      T* v = (T*)&raw;
#pragma unroll
      for (int i = 0; i < V; ++i) v[i] = times_p<T>(v[i], P);
      ((uint4*)out)[g] = raw;
    }
  } else {
    for (int d = threadIdx.x; d < D; d += 256) out[d] = times_p<T>(in[d], P);
  }
}

// out[d][e*P + p] = in[d][e]
template <typename T>
__global__ void transform_wg_kernel(const T* __restrict__ wg, T* __restrict__ out, int D, int E, int P) {
  const int64_t n = (int64_t)D * E * P;
  const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (q >= n) return;
  const int64_t d = q / ((int64_t)E * P);
  const int ep = (int)(q - d * E * P);
  out[q] = wg[d * E + ep / P];
}

static bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

template <typename T>
static hipError_t transform_all(const Layout& L, const void* wg, const void* w1, const void* w3, const void* w2,
                                const int32_t* perm, void* wg_out, void* w1_out, void* w3_out, void* w2_out, hipStream_t s) {
  constexpr int V = 16 / sizeof(T);
  const size_t lds = (size_t)2 * L.F * sizeof(T);
  const bool vec13 = L.Fp % V == 0 && lds <= 128 * 1024 && aligned16(w1) && aligned16(w3) && aligned16(w1_out) && aligned16(w3_out);
  hipError_t e;
  if (vec13) {
    e = hipFuncSetAttribute((const void*)transform_w13_lds_kernel<T>, hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);
    if (e != hipSuccess) return e;
    transform_w13_lds_kernel<T><<<dim3(L.D, L.E_res), dim3(256), lds, s>>>((const T*)w1, (const T*)w3, perm, (T*)w1_out,
                                                                           (T*)w3_out, L.D, L.F, L.P);
  } else {
    transform_w13_kernel<T><<<dim3(L.D, L.E_res), dim3(256), 0, s>>>((const T*)w1, (const T*)w3, perm, (T*)w1_out, (T*)w3_out,
                                                                     L.D, L.F, L.P);
  }
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (L.D % V == 0 && aligned16(w2) && aligned16(w2_out))
    transform_w2_kernel<T, true><<<dim3(L.F, L.E_res), dim3(256), 0, s>>>((const T*)w2, perm, (T*)w2_out, L.D, L.F, L.P);
  else
    transform_w2_kernel<T, false><<<dim3(L.F, L.E_res), dim3(256), 0, s>>>((const T*)w2, perm, (T*)w2_out, L.D, L.F, L.P);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (wg) {
    const int64_t n = (int64_t)L.D * L.E * L.P;
    transform_wg_kernel<T><<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s>>>((const T*)wg, (T*)wg_out, L.D, L.E, L.P);
    e = hipGetLastError();
  }
  return e;
}

hipError_t launch_transform_complete(const Layout& L, const void* wg, const void* w1, const void* w3, const void* w2,
                                     const int32_t* perm, void* wg_out, void* w1_out, void* w3_out, void* w2_out,
                                     hipStream_t s) {
  if (L.dtype == DSMOE_F32) return transform_all<float>(L, wg, w1, w3, w2, perm, wg_out, w1_out, w3_out, w2_out, s);
  return transform_all<uint16_t>(L, wg, w1, w3, w2, perm, wg_out, w1_out, w3_out, w2_out, s);
}

}  // namespace dsmoe
