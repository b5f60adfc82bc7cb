// bf16 MFMA grouped GEMMs for gfx950 (the hot loops of the layer).
//
//   GEMM-1  H[row][p*Fp + j] = Swish(x_row . W1[:, j]) * (x_row . W3[:, j])   (Eq. 4: gate, up, Swish*mul)
//           one work item = 256 rows (token-expert pairs of one expert) x 128 neurons of partition p
//   GEMM-2  Yp[row][d] = sum over the partitions p kept by some row of the tile, sum_j H[row][p*Fp+j] W2[p*Fp+j][d]
//           one work item = 256 rows x 256 output columns; dropped partitions are skipped whole
//
// Both kernels: 256 threads = 4 wavefronts in a 2 x 2 grid, each wavefront owns a 128 x 128 block
// of the 256 x 256 tile as 4 x 4 v_mfma_f32_32x32x16_bf16 accumulators (fp32).  Operand tiles
// [256][64] bf16 are brought HBM -> LDS with buffer loads that write LDS directly, double
// buffered (2 x 64 KiB of the CU's 160 KiB LDS).  Weight tiles are stored pre-swizzled by
// moe_partition_weights, so their copy is a linear 32 KiB stream; activation rows are gathered
// through the row list (GEMM-1) or read in place (GEMM-2) with the same chunk rotation.
#include "common.h"

namespace dsmoe {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((address_space(3))) void lds_void;

constexpr int kLdsBytes = 4 * kStageBytes;  // 2 buffers x (A tile + B tile) = 128 KiB
constexpr uint32_t kRsrcFlags = 0x00020000u;  // raw buffer, 32-bit elements

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, kRsrcFlags);
}

// 16 bytes per lane from (rsrc base + voff + soff) into LDS at (lds_uniform + lane * 16)
__device__ __forceinline__ void load16_to_lds(__amdgpu_buffer_rsrc_t rsrc, char* lds_uniform, uint32_t voff, uint32_t soff) {
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void*)lds_uniform, 16, voff, soff, 0, 0);
}

// XCD-aware order: consecutive block ids land on different XCDs (round robin over 8), so give
// each XCD a run of 32 consecutive work items out of every 256: items that share a weight tile
// then share an L2.
__device__ __forceinline__ int xcd_remap(int b) {
  const int chunk = b >> 8, within = b & 255;
  return (chunk << 8) + ((within & 7) << 5) + (within >> 3);
}

// One K step of the 256 x 256 tile for this wavefront: A rows wm*128.., B rows wn*128..
__device__ __forceinline__ void mma_step(const char* ldsA, const char* ldsB, int wm, int wn, int lane, f32x16 (&acc)[4][4]) {
  const int r32 = lane & 31, half = lane >> 5;
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    bf16x8 a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int ra = wm * 128 + i * 32 + r32;
      a[i] = *(const bf16x8*)(ldsA + ra * 128 + swz_chunk(ra, s * 2 + half) * 16);
      const int rb = wn * 128 + i * 32 + r32;
      b[i] = *(const bf16x8*)(ldsB + rb * 128 + swz_chunk(rb, s * 2 + half) * 16);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
  }
}

// ------------------------------------------------------------------------------------- GEMM-1
__global__ __launch_bounds__(256) void gemm1_mfma_kernel(Layout L, int T, const char* packed, const uint16_t* x, char* ws) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int32_t* counters = (const int32_t*)(ws + L.o_counters);
  const int item_id = xcd_remap(blockIdx.x);
  if (item_id >= counters[0]) return;
  const Item1 it = ((const Item1*)(ws + L.o_items1))[item_id];
  const int32_t* row_token = (const int32_t*)(ws + L.o_row_token);
  const uint8_t* row_bits = (const uint8_t*)(ws + L.o_row_bits);
  const bool sh = it.e == L.E_res;
  const int KS1 = L.D / kBK;
  const int Fp = sh ? L.F_shT : L.Fp;
  const int ld = sh ? L.F_shT : L.F;
  const char* wbase = sh ? packed + L.p_sw13 + (int64_t)it.jt * KS1 * kStageBytes
                         : packed + L.p_w13 + (((int64_t)it.e * L.P + it.p) * L.NT1 + it.jt) * KS1 * kStageBytes;
  const __amdgpu_buffer_rsrc_t rsW = make_rsrc(wbase, (uint32_t)(KS1 * kStageBytes));
  const __amdgpu_buffer_rsrc_t rsX = make_rsrc(x, (uint32_t)((int64_t)T * L.D * 2));

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int wm = w >> 1, wn = w & 1;
  // activation gather: this thread copies chunk (tid & 7) of rows i*32 + (tid >> 3)
  uint32_t xoff[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int r = i * 32 + (tid >> 3);
    const int rr = r < it.nrows ? r : it.nrows - 1;  // rows past the end re-read the last valid row
    const int tok = row_token[it.row0 + rr];
    xoff[i] = (uint32_t)tok * (uint32_t)(L.D * 2) + (uint32_t)(swz_chunk(r, tid & 7) * 16);
  }
  const uint32_t woff = (uint32_t)tid * 16;
  char* lds_w = lds + w * 1024;  // this wavefront's 1 KiB slice of every 4 KiB slab

  auto issue = [&](int ks, int buf) {
    char* la = lds_w + buf * (2 * kStageBytes);
    char* lb = la + kStageBytes;
#pragma unroll
    for (int i = 0; i < 8; ++i) load16_to_lds(rsW, la + i * 4096, woff, (uint32_t)(ks * kStageBytes + i * 4096));
#pragma unroll
    for (int i = 0; i < 8; ++i) load16_to_lds(rsX, lb + i * 4096, xoff[i], (uint32_t)(ks * (kBK * 2)));
  };

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  issue(0, 0);
  for (int ks = 0; ks < KS1; ++ks) {
    __syncthreads();  // stage ks has landed (all waves' loads), buffer (ks+1)&1 is free
    if (ks + 1 < KS1) issue(ks + 1, (ks + 1) & 1);
    const char* la = lds + (ks & 1) * (2 * kStageBytes);
    mma_step(la, la + kStageBytes, wm, wn, lane, acc);
  }

  // epilogue: MFMA A = weight rows (gate rows 0..63, up rows 64..127 of this wave), B = pair rows.
  // acc[i][j][v]: weight row i*32 + 8*(v/4) + 4*(lane/32) + v%4, pair row wn*128 + j*32 + lane%32.
  uint16_t* H = sh ? (uint16_t*)(ws + L.o_Hs) : (uint16_t*)(ws + L.o_H);
  const int hrow0 = sh ? it.row0 : it.row0 - L.sh_rows;
  const int nbase = it.jt * kMfmaNeur + wm * 64;  // first neuron (inside the partition) of this wave
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int r = wn * 128 + j * 32 + (lane & 31);
    if (r >= it.nrows) continue;
    const bool kept = (row_bits[it.row0 + r] >> it.p) & 1;
    uint16_t* hrow = H + (size_t)(hrow0 + r) * ld + (size_t)it.p * Fp;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
      for (int vq = 0; vq < 4; ++vq) {
        const int n0 = nbase + i * 32 + vq * 8 + (lane >> 5) * 4;
        if (n0 >= Fp) continue;
        uint16_t o[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const float g = acc[i][j][vq * 4 + c], u = acc[i + 2][j][vq * 4 + c];
          o[c] = kept ? f32_to_bf16(silu_fast(g) * u) : (uint16_t)0;
        }
        uint2 pk;
        pk.x = o[0] | ((uint32_t)o[1] << 16);
        pk.y = o[2] | ((uint32_t)o[3] << 16);
        *(uint2*)(hrow + n0) = pk;
      }
    }
  }
}

// ------------------------------------------------------------------------------------- GEMM-2
__global__ __launch_bounds__(256) void gemm2_mfma_kernel(Layout L, int T, const char* packed, char* ws) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int32_t* counters = (const int32_t*)(ws + L.o_counters);
  const int item_id = xcd_remap(blockIdx.x);
  if (item_id >= counters[1]) return;
  const Item2 it = ((const Item2*)(ws + L.o_items2))[item_id];
  const bool sh = it.e == L.E_res;
  const int Fp = sh ? L.F_shT : L.Fp;
  const int ld = sh ? L.F_shT : L.F;
  const int KT = ld / kBK;        // K steps of the whole expert
  const int KSp = Fp / kBK;       // K steps of one partition
  const char* wbase = sh ? packed + L.p_sw2 + (int64_t)it.jd * KT * kStageBytes
                         : packed + L.p_w2 + ((int64_t)it.e * L.ND2 + it.jd) * KT * kStageBytes;
  const uint16_t* H = sh ? (const uint16_t*)(ws + L.o_Hs) : (const uint16_t*)(ws + L.o_H);
  const int hrow0 = sh ? it.row0 : it.row0 - L.sh_rows;
  const char* hbase = (const char*)(H + (size_t)hrow0 * ld);
  const __amdgpu_buffer_rsrc_t rsW = make_rsrc(wbase, (uint32_t)((int64_t)KT * kStageBytes));
  const __amdgpu_buffer_rsrc_t rsH = make_rsrc(hbase, (uint32_t)((int64_t)it.nrows * ld * 2));

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int wm = w >> 1, wn = w & 1;
  uint32_t hoff[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int r = i * 32 + (tid >> 3);
    const int rr = r < it.nrows ? r : it.nrows - 1;
    hoff[i] = (uint32_t)rr * (uint32_t)(ld * 2) + (uint32_t)(swz_chunk(r, tid & 7) * 16);
  }
  const uint32_t woff = (uint32_t)tid * 16;
  char* lds_w = lds + w * 1024;

  auto issue = [&](int kt, int buf) {  // kt = K step in the expert's neuron positions
    char* la = lds_w + buf * (2 * kStageBytes);
    char* lb = la + kStageBytes;
#pragma unroll
    for (int i = 0; i < 8; ++i) load16_to_lds(rsH, la + i * 4096, hoff[i], (uint32_t)(kt * (kBK * 2)));
#pragma unroll
    for (int i = 0; i < 8; ++i) load16_to_lds(rsW, lb + i * 4096, woff, (uint32_t)(kt * kStageBytes + i * 4096));
  };

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // K steps run over the partitions some row of this tile keeps (Sec. 4: dropped units cost nothing)
  const int np = sh ? 1 : L.P;
  int nsteps = 0;
  for (int p = 0; p < np; ++p) nsteps += ((it.kmask >> p) & 1) ? KSp : 0;
  // step -> kt: walk the kept partitions in order
  int p_cur = 0, k_in = 0;
  auto advance_to_kept = [&]() {
    while (p_cur < np && !((it.kmask >> p_cur) & 1)) ++p_cur;
  };
  advance_to_kept();
  auto next_kt = [&]() {
    int kt = p_cur * KSp + k_in;
    if (++k_in == KSp) {
      k_in = 0;
      ++p_cur;
      advance_to_kept();
    }
    return kt;
  };
  if (nsteps > 0) issue(next_kt(), 0);
  for (int st = 0; st < nsteps; ++st) {
    __syncthreads();
    if (st + 1 < nsteps) issue(next_kt(), (st + 1) & 1);
    const char* la = lds + (st & 1) * (2 * kStageBytes);
    mma_step(la, la + kStageBytes, wm, wn, lane, acc);
  }

  // epilogue: acc[i][j][v]: pair row wm*128 + i*32 + 8*(v/4) + 4*(lane/32) + v%4, column wn*128 + j*32 + lane%32
  float* Yp = (float*)(ws + L.o_Yp);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int r = wm * 128 + i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
      if (r >= it.nrows) continue;
      float* yrow = Yp + (size_t)(it.row0 + r) * L.D + it.jd * kMfmaBN2;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int c = wn * 128 + j * 32 + (lane & 31);
        if (it.jd * kMfmaBN2 + c < L.D) yrow[c] = acc[i][j][v];
      }
    }
  }
}

static hipError_t set_lds_attr() {
  static bool attr_set = false;
  if (attr_set) return hipSuccess;
  hipError_t e = hipFuncSetAttribute((const void*)gemm1_mfma_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
  if (e != hipSuccess) return e;
  e = hipFuncSetAttribute((const void*)gemm2_mfma_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
  if (e != hipSuccess) return e;
  attr_set = true;
  return hipSuccess;
}

// grids are whole chunks of 256 blocks so that the XCD remap is a bijection
hipError_t launch_gemm1_mfma(const Layout& L, int T, const char* packed, const void* x, char* ws, hipStream_t s) {
  if (T <= 0) return hipSuccess;
  hipError_t e = set_lds_attr();
  if (e != hipSuccess) return e;
  const int g1 = (items1_bound(L, T) + 255) & ~255;
  gemm1_mfma_kernel<<<dim3(g1), dim3(256), kLdsBytes, s>>>(L, T, packed, (const uint16_t*)x, ws);
  return hipGetLastError();
}

hipError_t launch_gemm2_mfma(const Layout& L, int T, const char* packed, char* ws, hipStream_t s) {
  if (T <= 0) return hipSuccess;
  hipError_t e = set_lds_attr();
  if (e != hipSuccess) return e;
  const int g2 = (items2_bound(L, T) + 255) & ~255;
  gemm2_mfma_kernel<<<dim3(g2), dim3(256), kLdsBytes, s>>>(L, T, packed, ws);
  return hipGetLastError();
}

}  // namespace dsmoe
