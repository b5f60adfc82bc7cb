// Gating logits l = x W_g (Sec. 3.1 of the paper, first equation; W_g is [d_model][E]): the small
// product in front of the softmax of Eq. 1.  HBM-bound: x is read once, W_g stays in L2.
//
// bf16 layers with d_model % 64 == 0 use the matrix cores.  W_g is repacked once into MFMA operand
// order, so a lane fetches its 8 values of an operand with one 16-byte load and a wavefront reads
// 1 KiB contiguous per operand.  A lane reads 64 contiguous bytes of its token per step (a wavefront
// covers whole 128-byte lines of 32 tokens) and feeds four MFMAs with them: the contraction index
// is walked in the order (64-step, lane half, MFMA, 8 values), which x and the packed W_g share.
#include "common.h"

namespace dsmoe {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int kRouterStep = 64;    // contraction values per step
constexpr int kRouterTokens = 32;  // tokens per workgroup

// packed W_g, MFMA path: chunk ((ks*4 + m)*NT + nt)*64 + lane holds W_g[ks*64 + (lane/32)*32 + m*8 + i][nt*32 + lane%32],
// i = 0..7 (zero for experts >= E).  One thread per chunk.
__global__ void router_pack_mfma_kernel(const uint16_t* __restrict__ wg, uint16_t* __restrict__ out, int D, int E, int NT) {
  const int64_t total = (int64_t)(D / kRouterStep) * 4 * NT * 64;
  const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (q >= total) return;
  const int lane = (int)(q & 63);
  int64_t r = q >> 6;
  const int nt = (int)(r % NT);
  r /= NT;
  const int m = (int)(r & 3);
  const int ks = (int)(r >> 2);
  const int e = nt * 32 + (lane & 31);
  const int d0 = ks * kRouterStep + (lane >> 5) * 32 + m * 8;
  for (int i = 0; i < 8; ++i) out[q * 8 + i] = e < E ? wg[(size_t)(d0 + i) * E + e] : (uint16_t)0;
}

// generic path: W_g widened to float, same [D][E] layout
template <typename T>
__global__ void router_pack_generic_kernel(const T* __restrict__ wg, float* __restrict__ out, int64_t n) {
  const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (q >= n) return;
  if constexpr (sizeof(T) == 2) out[q] = bf16_to_f32(wg[q]);
  else out[q] = wg[q];
}

// Workgroup = 32 tokens x (NT tiles of 32 experts); its W wavefronts take every W-th 64-step of the
// contraction (enough loads in flight to stream x at HBM rate even for a few thousand tokens) and
// add their partial tiles through LDS in a fixed order, so results are reproducible bit for bit.
template <int NT, int W>
__global__ __launch_bounds__(W * 64) void router_mfma_kernel(const uint16_t* __restrict__ x, const uint4* __restrict__ wgp,
                                                             float* __restrict__ logits, int T, int D, int E, int NT_all) {
  extern __shared__ float part[];  // [W][NT][16][64]: wavefront, tile, accumulator register, lane
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int t0 = blockIdx.x * kRouterTokens;
  const int nt0 = blockIdx.y * NT;
  const int trow = min(t0 + (lane & 31), T - 1);  // rows past the end re-read the last token; not stored
  const uint4* xa = (const uint4*)(x + (size_t)trow * D + (lane >> 5) * 32);
  const int KS = D / kRouterStep;
  f32x16 acc[NT];
#pragma unroll
  for (int j = 0; j < NT; ++j)
    for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
  int tile[NT];
#pragma unroll
  for (int j = 0; j < NT; ++j) tile[j] = min(nt0 + j, NT_all - 1);  // a group's tiles past the end repeat the last one; not stored
  for (int ks = w; ks < KS; ks += W) {
    uint4 a[4];
#pragma unroll
    for (int m = 0; m < 4; ++m) a[m] = xa[ks * 8 + m];
#pragma unroll
    for (int m = 0; m < 4; ++m) {
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        const uint4 b = wgp[((size_t)(ks * 4 + m) * NT_all + tile[j]) * 64 + lane];
        acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[m]), __builtin_bit_cast(bf16x8, b), acc[j], 0, 0, 0);
      }
    }
  }
#pragma unroll
  for (int j = 0; j < NT; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) part[((w * NT + j) * 16 + v) * 64 + lane] = acc[j][v];
  __syncthreads();
  // value (j, v, l): token t0 + 8*(v/4) + 4*(l/32) + v%4, expert (nt0+j)*32 + l%32
  for (int o = tid; o < NT * 1024; o += W * 64) {
    const int j = o >> 10, v = (o >> 6) & 15, l = o & 63;
    float sum = 0.f;
    for (int ww = 0; ww < W; ++ww) sum += part[((ww * NT + j) * 16 + v) * 64 + l];
    const int e = (nt0 + j) * 32 + (l & 31);
    const int t = t0 + 8 * (v >> 2) + 4 * (l >> 5) + (v & 3);
    if (nt0 + j < NT_all && e < E && t < T) logits[(size_t)t * E + e] = sum;
  }
}

// generic path: a wavefront per token, lanes stride over d_model, experts in chunks of 8
template <typename T>
__global__ __launch_bounds__(256) void router_generic_kernel(const T* __restrict__ x, const float* __restrict__ wgf,
                                                             float* __restrict__ logits, int Tn, int D, int E) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= Tn) return;
  for (int e0 = 0; e0 < E; e0 += 8) {
    float acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0.f;
    for (int d = lane; d < D; d += 64) {
      float xv;
      if constexpr (sizeof(T) == 2) xv = bf16_to_f32(x[(size_t)t * D + d]);
      else xv = x[(size_t)t * D + d];
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (e0 + j < E) acc[j] = fmaf(xv, wgf[(size_t)d * E + e0 + j], acc[j]);
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float v = acc[j];
      for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
      if (lane == 0 && e0 + j < E) logits[(size_t)t * E + e0 + j] = v;
    }
  }
}

hipError_t launch_router_pack(const Layout& L, const void* wg, char* out, hipStream_t s) {
  if (L.router_mfma) {
    const int NT = (L.E + 31) / 32;
    const int64_t total = (int64_t)(L.D / kRouterStep) * 4 * NT * 64;
    router_pack_mfma_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s>>>((const uint16_t*)wg, (uint16_t*)out, L.D,
                                                                                        L.E, NT);
  } else {
    const int64_t n = (int64_t)L.D * L.E;
    const dim3 grid((unsigned)((n + 255) / 256));
    if (L.dtype == DSMOE_F32) router_pack_generic_kernel<float><<<grid, dim3(256), 0, s>>>((const float*)wg, (float*)out, n);
    else router_pack_generic_kernel<uint16_t><<<grid, dim3(256), 0, s>>>((const uint16_t*)wg, (float*)out, n);
  }
  return hipGetLastError();
}

template <int NT, int W>
static hipError_t launch_router_mfma(const Layout& L, int T, const uint4* wgp, const void* x, float* logits, int NT_all,
                                     hipStream_t s) {
  constexpr int lds = W * NT * 16 * 64 * 4;
  static PerDeviceOnce once;  // one per instantiation
  hipError_t e = once.run([] { return hipFuncSetAttribute((const void*)router_mfma_kernel<NT, W>, hipFuncAttributeMaxDynamicSharedMemorySize, lds); });
  if (e != hipSuccess) return e;
  const dim3 grid((unsigned)((T + kRouterTokens - 1) / kRouterTokens), (unsigned)((NT_all + NT - 1) / NT));
  router_mfma_kernel<NT, W><<<grid, dim3(W * 64), lds, s>>>((const uint16_t*)x, wgp, logits, T, L.D, L.E, NT_all);
  return hipGetLastError();
}

hipError_t launch_router(const Layout& L, int T, const char* router_packed, const void* x, float* logits, hipStream_t s) {
  if (T <= 0) return hipSuccess;
  if (L.router_mfma) {
    const int NT = (L.E + 31) / 32;
    const uint4* wgp = (const uint4*)router_packed;
    if (NT == 1) return launch_router_mfma<1, 16>(L, T, wgp, x, logits, NT, s);
    if (NT == 2) return launch_router_mfma<2, 16>(L, T, wgp, x, logits, NT, s);
    return launch_router_mfma<4, 8>(L, T, wgp, x, logits, NT, s);
  } else {
    const dim3 grid((unsigned)((T + 3) / 4));
    if (L.dtype == DSMOE_F32) router_generic_kernel<float><<<grid, dim3(256), 0, s>>>((const float*)x, (const float*)router_packed, logits, T, L.D, L.E);
    else router_generic_kernel<uint16_t><<<grid, dim3(256), 0, s>>>((const uint16_t*)x, (const float*)router_packed, logits, T, L.D, L.E);
  }
  return hipGetLastError();
}

}  // namespace dsmoe
