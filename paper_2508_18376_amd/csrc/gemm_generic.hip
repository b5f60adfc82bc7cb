// Generic grouped GEMM path: fp32 accumulation on the vector ALUs, any D and F/P.
// Used for fp32 layers (where it is the full-precision path) and for bf16 layers whose shape the
// MFMA kernels do not cover.  The intermediate activation H is fp32 here whatever the layer's type.  Same work lists, same row lists, same math as the MFMA path:
//   GEMM-1  H[row][p*Fp + j] = Swish(x_row . W1[:, j]) * (x_row . W3[:, j])      (Eq. 4, gate/up)
//   GEMM-2  Yp[row][d] = sum over kept partitions p, neurons j of H[row][p*Fp+j] * W2[p*Fp+j][d]
// with the neurons already in permuted order (Sec. 4.2 b) and split into P slices (Sec. 3.2).
#include "common.h"

namespace dsmoe {

template <typename T>
__device__ __forceinline__ float ldf(const T* p, size_t i);
template <>
__device__ __forceinline__ float ldf<float>(const float* p, size_t i) { return p[i]; }
template <>
__device__ __forceinline__ float ldf<uint16_t>(const uint16_t* p, size_t i) { return bf16_to_f32(p[i]); }
template <typename T>
__device__ __forceinline__ void stf(T* p, size_t i, float v);
template <>
__device__ __forceinline__ void stf<float>(float* p, size_t i, float v) { p[i] = v; }
template <>
__device__ __forceinline__ void stf<uint16_t>(uint16_t* p, size_t i, float v) { p[i] = f32_to_bf16(v); }

constexpr int GK = 16;  // K step

template <typename T>
__global__ __launch_bounds__(256) void gemm1_generic_kernel(Layout L, const char* packed, const T* x, char* ws, int epi) {
  const int32_t* counters = (const int32_t*)(ws + L.o_counters);
  if ((int)blockIdx.x >= counters[0]) return;
  const Item1 it = ((const Item1*)(ws + L.o_items1))[blockIdx.x];
  const int32_t* row_token = (const int32_t*)(ws + L.o_row_token);
  const uint8_t* row_bits = (const uint8_t*)(ws + L.o_row_bits);
  const bool sh = it.e == L.E_res;
  const int ld = sh ? L.F_shT : L.F;         // neurons of the expert = row length of W1/W3/H
  const int Fp = sh ? L.F_shT : L.Fp;
  const int col0 = it.p * Fp + it.jt * kGenBN;
  const int ncols = min(kGenBN, Fp - it.jt * kGenBN);
  const T* w1 = sh ? (const T*)(packed + L.p_sw13) : (const T*)(packed + L.p_w13) + (size_t)it.e * L.D * L.F;
  const T* w3 = w1 + (sh ? (size_t)L.D * L.F_shT : (size_t)L.E_res * L.D * L.F);
  float* H = sh ? (float*)(ws + L.o_Hs) : (float*)(ws + L.o_H);
  const int hrow0 = sh ? it.row0 : it.row0 - L.sh_rows;

  __shared__ float As[GK][kGenBM + 1];
  __shared__ float B1[GK][kGenBN + 1];
  __shared__ float B3[GK][kGenBN + 1];
  const int tid = threadIdx.x, ty = tid / 16, tx = tid % 16;
  float a1[4][4] = {}, a3[4][4] = {};
  for (int k0 = 0; k0 < L.D; k0 += GK) {
    for (int i = 0; i < 4; ++i) {
      int q = tid + i * 256;
      int r = q / GK, kk = q % GK;
      float v = 0.f;
      if (r < it.nrows && k0 + kk < L.D) v = ldf<T>(x, (size_t)row_token[it.row0 + r] * L.D + k0 + kk);
      As[kk][r] = v;
      int kb = q / kGenBN, c = q % kGenBN;
      float b1 = 0.f, b3 = 0.f;
      if (c < ncols && k0 + kb < L.D) {
        size_t o = (size_t)(k0 + kb) * ld + col0 + c;
        b1 = ldf<T>(w1, o);
        b3 = ldf<T>(w3, o);
      }
      B1[kb][c] = b1;
      B3[kb][c] = b3;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < GK; ++kk) {
      float av[4], g[4], u[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) av[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        g[j] = B1[kk][tx * 4 + j];
        u[j] = B3[kk][tx * 4 + j];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          a1[i][j] = fmaf(av[i], g[j], a1[i][j]);
          a3[i][j] = fmaf(av[i], u[j], a3[i][j]);
        }
    }
    __syncthreads();
  }
  for (int i = 0; i < 4; ++i) {
    int r = ty * 4 + i;
    if (r >= it.nfill) continue;  // rows [nrows, nfill) keep nothing of this partition: zeros
    bool kept = r < it.nrows && ((row_bits[it.row0 + r] >> it.p) & 1);
    for (int j = 0; j < 4; ++j) {
      int c = tx * 4 + j;
      if (c >= ncols) continue;
      float h = kept ? epi_value<false>(epi, a1[i][j], a3[i][j]) : 0.f;
      H[(size_t)(hrow0 + r) * ld + col0 + c] = h;
    }
  }
}

template <typename T>
__global__ __launch_bounds__(256) void gemm2_generic_kernel(Layout L, const char* packed, char* ws) {
  const int32_t* counters = (const int32_t*)(ws + L.o_counters);
  if ((int)blockIdx.x >= counters[1]) return;
  const Item2 it = ((const Item2*)(ws + L.o_items2))[blockIdx.x];
  const bool sh = it.e == L.E_res;
  const int ld = sh ? L.F_shT : L.F;
  const int Fp = sh ? L.F_shT : L.Fp;
  const T* w2 = sh ? (const T*)(packed + L.p_sw2) : (const T*)(packed + L.p_w2) + (size_t)it.e * L.F * L.D;
  const float* H = sh ? (const float*)(ws + L.o_Hs) : (const float*)(ws + L.o_H);
  const int hrow0 = sh ? it.row0 : it.row0 - L.sh_rows;
  float* Yp = (float*)(ws + L.o_Yp);
  const int d0 = it.jd * kGenBN;
  const int ncols = min(kGenBN, L.D - d0);

  __shared__ float As[GK][kGenBM + 1];
  __shared__ float Bs[GK][kGenBN + 1];
  const int tid = threadIdx.x, ty = tid / 16, tx = tid % 16;
  float acc[4][4] = {};
  const int np = sh ? 1 : L.P;
  for (int p = 0; p < np; ++p) {
    if (!((it.kmask >> p) & 1)) continue;  // no row of this tile keeps partition p
    for (int k0 = 0; k0 < Fp; k0 += GK) {
      for (int i = 0; i < 4; ++i) {
        int q = tid + i * 256;
        int r = q / GK, kk = q % GK;
        float v = 0.f;
        if (r < it.nrows && k0 + kk < Fp) v = H[(size_t)(hrow0 + r) * ld + p * Fp + k0 + kk];
        As[kk][r] = v;
        int kb = q / kGenBN, c = q % kGenBN;
        float b = 0.f;
        if (c < ncols && k0 + kb < Fp) b = ldf<T>(w2, (size_t)(p * Fp + k0 + kb) * L.D + d0 + c);
        Bs[kb][c] = b;
      }
      __syncthreads();
#pragma unroll
      for (int kk = 0; kk < GK; ++kk) {
        float av[4], bv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) av[i] = As[kk][ty * 4 + i];
#pragma unroll
        for (int j = 0; j < 4; ++j) bv[j] = Bs[kk][tx * 4 + j];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
      }
      __syncthreads();
    }
  }
  for (int i = 0; i < 4; ++i) {
    int r = ty * 4 + i;
    if (r >= it.nrows) continue;
    for (int j = 0; j < 4; ++j) {
      int c = tx * 4 + j;
      if (c < ncols) Yp[(size_t)(it.row0 + r) * L.D + d0 + c] = acc[i][j];
    }
  }
}

hipError_t launch_gemm1_generic(const Layout& L, int T, const char* packed, const void* x, char* ws, int epi, hipStream_t s) {
  if (T <= 0) return hipSuccess;
  dim3 block(256), grid(items1_bound(L, T));
  if (L.dtype == DSMOE_F32) gemm1_generic_kernel<float><<<grid, block, 0, s>>>(L, packed, (const float*)x, ws, epi);
  else gemm1_generic_kernel<uint16_t><<<grid, block, 0, s>>>(L, packed, (const uint16_t*)x, ws, epi);
  return hipGetLastError();
}

hipError_t launch_gemm2_generic(const Layout& L, int T, const char* packed, char* ws, hipStream_t s) {
  if (T <= 0) return hipSuccess;
  dim3 block(256), grid(items2_bound(L, T));
  if (L.dtype == DSMOE_F32) gemm2_generic_kernel<float><<<grid, block, 0, s>>>(L, packed, ws);
  else gemm2_generic_kernel<uint16_t><<<grid, block, 0, s>>>(L, packed, ws);
  return hipGetLastError();
}

}  // namespace dsmoe
