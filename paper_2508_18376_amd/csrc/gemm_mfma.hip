// bf16 MFMA grouped GEMMs for gfx950 (the hot loops of the layer).
//
//   GEMM-1  H[row][p*Fp + j] = Swish(x_row . W1[:, j]) * (x_row . W3[:, j])   (Eq. 4: gate, up, Swish*mul)
//           one work item = 256 rows (token-expert pairs of one expert) x 128 neurons of partition p
//   GEMM-2  Yp[row][d] = sum over the partitions p kept by some row of the tile, sum_j H[row][p*Fp+j] W2[p*Fp+j][d]
//           one work item = 256 rows x 256 output columns; dropped partitions are skipped whole
//
// Both kernels: 256 threads = 4 wavefronts in a 2 x 2 grid, each wavefront owns a 128 x 128 block
// of the 256 x 256 tile as 4 x 4 v_mfma_f32_32x32x16_bf16 accumulators (fp32, 256 registers).
// Operand tiles [256][32] bf16 travel HBM/L2 -> LDS by buffer loads that write LDS directly (no
// registers in between), through a ring of 4 stages (4 x 32 KiB of the CU's 160 KiB LDS), three
// stages in flight ahead of the one being multiplied.  Weight tiles are stored pre-swizzled by
// moe_partition_weights, so their copy is a linear 16 KiB stream; activation rows are gathered
// through the row list (GEMM-1) or read in place (GEMM-2) with the same chunk rotation.
//
// The loads are written as inline assembly so that their completion can be awaited per stage
// (s_waitcnt vmcnt(N)): the compiler never sees them and must not be allowed to move LDS reads
// across the hand-placed waits and barriers, which is what the "memory" clobbers are for.
#include "common.h"

namespace dsmoe {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(int)))) int i32x4;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;

constexpr int kStages = 4;                          // LDS ring depth
constexpr int kStagePair = 2 * kStageBytes;         // A tile + B tile of one stage: 32 KiB
constexpr int kLdsBytes = kStages * kStagePair;     // 128 KiB
constexpr int kLoadsPerStage = 2 * (kStageBytes / 16 / 256);  // per thread: 4 (A) + 4 (B)
constexpr uint32_t kRsrcFlags = 0x00020000u;        // raw buffer, 32-bit elements

__device__ __forceinline__ i32x4 make_rsrc(const void* base, uint32_t bytes) {
  // buffer descriptor: base address (48 bits), stride 0, size in bytes, format flags
  const uint64_t a = (uint64_t)(uintptr_t)base;
  i32x4 r;
  r[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)a);
  r[1] = __builtin_amdgcn_readfirstlane((int)(uint32_t)((a >> 32) & 0xffffu));
  r[2] = __builtin_amdgcn_readfirstlane((int)bytes);
  r[3] = (int)kRsrcFlags;
  return r;
}

// 16 bytes per lane from (rsrc base + voff + soff) straight into LDS at (lds_addr + lane * 16);
// lds_addr (byte address inside the workgroup's LDS) must be wave-uniform.
__device__ __forceinline__ void dma16(i32x4 rsrc, uint32_t lds_addr, uint32_t voff, uint32_t soff) {
  asm volatile(
      "s_mov_b32 m0, %0\n\t"
      "s_nop 0\n\t"
      "buffer_load_dwordx4 %1, %2, %3 offen lds"
      :
      : "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff)
      : "memory");
}

// byte offset of a __shared__ object inside the workgroup's LDS allocation (what M0 wants)
__device__ __forceinline__ uint32_t lds_offset(const char* p) {
  return (uint32_t)(uintptr_t)((__attribute__((address_space(3))) const char*)p);
}

template <int N>
__device__ __forceinline__ void wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
__device__ __forceinline__ void block_barrier() { asm volatile("s_barrier" ::: "memory"); }

// XCD-aware order: consecutive block ids land on different XCDs (round robin over 8), so give
// each XCD a run of 32 consecutive work items out of every 256: items that share a weight tile
// then share an L2.
__device__ __forceinline__ int xcd_remap(int b) {
  const int chunk = b >> 8, within = b & 255;
  return (chunk << 8) + ((within & 7) << 5) + (within >> 3);
}

struct Frags {
  bf16x8 a[4], b[4];
};

// operand fragments of K substep s (16 values of K) of one stage: A rows wm*128 + i*32 + lane%32
__device__ __forceinline__ void load_frags(Frags& f, const char* stage, uint32_t offA, uint32_t offB) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    f.a[i] = *(const bf16x8*)(stage + offA + i * (32 * kBK * 2));
    f.b[i] = *(const bf16x8*)(stage + kStageBytes + offB + i * (32 * kBK * 2));
  }
}

__device__ __forceinline__ void mma16(const Frags& f, f32x16 (&acc)[4][4]) {
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[i], f.b[j], acc[i][j], 0, 0, 0);
}

// interleave hint for one half stage: 16 MFMAs with 8 LDS reads spread between them
__device__ __forceinline__ void sched_half_stage() {
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);  // 2 MFMA
    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // 1 DS read
  }
}

// The pipelined main loop shared by both GEMMs.
//   begin(st): fix the ring slot and the K offsets of stage st (called once per stage, in order);
//   one(q):    enqueue this thread's q-th DMA load (0..kLoadsPerStage-1) of the stage begun last.
// On return every DMA has completed and acc holds the tile.
//
// Per stage a wavefront issues 32 MFMAs (1024 matrix-core cycles), 16 LDS reads and 8 DMA loads.
// With one wavefront per SIMD nothing else hides an instruction that stalls the stream, so the
// reads and loads are threaded between the MFMAs by hand and pinned with scheduling barriers.
template <class Begin, class One>
__device__ __forceinline__ void mainloop(int n, Begin&& begin, One&& one, const char* lds, int wm, int wn, int lane,
                                         f32x16 (&acc)[4][4]) {
  const int r32 = lane & 31, half = lane >> 5;
  const int sw = (r32 >> 2) & 3;
  // byte offsets inside a stage's A / B tile for substep 0 and 1
  const uint32_t rowA = (uint32_t)(wm * 128 + r32) * (kBK * 2), rowB = (uint32_t)(wn * 128 + r32) * (kBK * 2);
  const uint32_t c0 = (uint32_t)((half ^ sw) * 16), c1 = (uint32_t)(((2 + half) ^ sw) * 16);
  Frags f0, f1;
  if (n <= 0) return;
  auto issue_all = [&](int st) {
    begin(st);
#pragma unroll
    for (int q = 0; q < kLoadsPerStage; ++q) one(q);
  };
  issue_all(0);
  if (n > 1) issue_all(1);
  if (n > 2) issue_all(2);
  if (n > 2) wait_vm<2 * kLoadsPerStage>();
  else if (n > 1) wait_vm<kLoadsPerStage>();
  else wait_vm<0>();
  block_barrier();
  load_frags(f0, lds, rowA + c0, rowB + c0);

  // first half of a stage: multiply substep 0 while the substep 1 operands stream in from LDS
  auto first_half = [&](int st) {
    const char* cur = lds + (st % kStages) * kStagePair;
    load_frags(f1, cur, rowA + c1, rowB + c1);
    mma16(f0, acc);
    sched_half_stage();
    __builtin_amdgcn_sched_barrier(0);
  };
  int st = 0;
  for (; st + 3 < n; ++st) {
    first_half(st);
    // stage st+1 must have landed for every wave (st+2 may still be in flight); after the barrier
    // every wave has also finished reading stage st-1, whose slot stage st+3 takes
    wait_vm<kLoadsPerStage>();
    block_barrier();
    begin(st + 3);
    // second half: multiply substep 1; between the MFMAs, enqueue stage st+3 and fetch substep 0 of stage st+1
    const char* nxt = lds + ((st + 1) % kStages) * kStagePair;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      acc[i][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f1.a[i], f1.b[0], acc[i][0], 0, 0, 0);
      acc[i][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f1.a[i], f1.b[1], acc[i][1], 0, 0, 0);
      one(2 * i);
      f0.a[i] = *(const bf16x8*)(nxt + rowA + c0 + i * (32 * kBK * 2));
      __builtin_amdgcn_sched_barrier(0);
      acc[i][2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f1.a[i], f1.b[2], acc[i][2], 0, 0, 0);
      acc[i][3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f1.a[i], f1.b[3], acc[i][3], 0, 0, 0);
      one(2 * i + 1);
      f0.b[i] = *(const bf16x8*)(nxt + kStageBytes + rowB + c0 + i * (32 * kBK * 2));
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  for (; st + 1 < n; ++st) {  // last stages: nothing left to enqueue
    first_half(st);
    if (st + 2 < n) wait_vm<kLoadsPerStage>();
    else wait_vm<0>();
    block_barrier();
    const char* nxt = lds + ((st + 1) % kStages) * kStagePair;
    load_frags(f0, nxt, rowA + c0, rowB + c0);
    mma16(f1, acc);
    sched_half_stage();
    __builtin_amdgcn_sched_barrier(0);
  }
  const char* last = lds + ((n - 1) % kStages) * kStagePair;
  load_frags(f1, last, rowA + c1, rowB + c1);
  mma16(f0, acc);
  mma16(f1, acc);
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
  const i32x4 rsW = make_rsrc(wbase, (uint32_t)(KS1 * kStageBytes));
  const i32x4 rsX = make_rsrc(x, (uint32_t)((int64_t)T * L.D * 2));

  const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = w >> 1, wn = w & 1;
  // activation gather: this thread copies chunk (tid & 3) of rows i*64 + (tid >> 2)
  uint32_t xoff[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = i * 64 + (tid >> 2);
    const int rr = r < it.nrows ? r : it.nrows - 1;  // rows past the end re-read the last valid row
    const int tok = row_token[it.row0 + rr];
    xoff[i] = (uint32_t)tok * (uint32_t)(L.D * 2) + (uint32_t)(swz_chunk(r, tid & 3) * 16);
  }
  const uint32_t woff = (uint32_t)tid * 16;
  // LDS byte address of this wavefront's 1 KiB slice of each 4 KiB slab
  const uint32_t lds_w = lds_offset(lds) + (uint32_t)(w * 1024);

  uint32_t slot = 0, sW = 0, sX = 0;
  auto begin = [&](int st) {
    slot = (uint32_t)(st % kStages) * kStagePair + lds_w;
    sW = (uint32_t)(st * kStageBytes);
    sX = (uint32_t)(st * (kBK * 2));
  };
  auto one = [&](int q) {
    if (q < 4) dma16(rsW, slot + q * 4096, woff, sW + q * 4096);
    else dma16(rsX, slot + kStageBytes + (q - 4) * 4096, xoff[q - 4], sX);
  };

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  mainloop(KS1, begin, one, lds, wm, wn, lane, acc);

  // epilogue: MFMA A = weight rows (gate rows 0..63, up rows 64..127 of this wave), B = pair rows.
  // acc[i][j][v]: weight row i*32 + 8*(v/4) + 4*(lane/32) + v%4, pair row wn*128 + j*32 + lane%32.
  // Swish(gate) * up is rounded to bf16 and parked in LDS as a [256 rows][128 neurons] tile
  // (rows padded to 272 bytes against bank conflicts), then written out in whole 256-byte row
  // segments: 16 lanes per row, 16 bytes per lane.
  constexpr int kHsRow = kMfmaNeur * 2 + 16;
  block_barrier();  // every wave is done reading the last stage
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int r = wn * 128 + j * 32 + (lane & 31);
    const bool kept = r < it.nrows && ((row_bits[it.row0 + (r < it.nrows ? r : 0)] >> it.p) & 1);
    char* srow = lds + r * kHsRow + (wm * 64 + (lane >> 5) * 4) * 2;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
      for (int vq = 0; vq < 4; ++vq) {
        bf16x2 lo, hi;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const float g = acc[i][j][vq * 4 + c], u = acc[i + 2][j][vq * 4 + c];
          const float h = kept ? g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)) * u : 0.f;  // Swish(g) * u, Eq. 4
          if (c < 2) lo[c] = (__bf16)h;
          else hi[c - 2] = (__bf16)h;
        }
        uint2 pk;
        pk.x = __builtin_bit_cast(uint32_t, lo);
        pk.y = __builtin_bit_cast(uint32_t, hi);
        *(uint2*)(srow + (i * 32 + vq * 8) * 2) = pk;
      }
    }
  }
  __syncthreads();
  uint16_t* H = sh ? (uint16_t*)(ws + L.o_Hs) : (uint16_t*)(ws + L.o_H);
  const int hrow0 = sh ? it.row0 : it.row0 - L.sh_rows;
  const int n_in = it.jt * kMfmaNeur + (tid & 15) * 8;  // first of this lane's 8 neurons, inside the partition
  if (n_in < Fp) {
#pragma unroll 4
    for (int c = 0; c < 16; ++c) {
      const int r = c * 16 + (tid >> 4);
      if (r < it.nrows) {
        const uint4 v = *(const uint4*)(lds + r * kHsRow + (tid & 15) * 16);
        *(uint4*)(H + (size_t)(hrow0 + r) * ld + (size_t)it.p * Fp + n_in) = v;
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
  const int KT = ld / kBK;        // stages of the whole expert
  const int KSp = Fp / kBK;       // stages of one partition
  const char* wbase = sh ? packed + L.p_sw2 + (int64_t)it.jd * KT * kStageBytes
                         : packed + L.p_w2 + ((int64_t)it.e * L.ND2 + it.jd) * KT * kStageBytes;
  const uint16_t* H = sh ? (const uint16_t*)(ws + L.o_Hs) : (const uint16_t*)(ws + L.o_H);
  const int hrow0 = sh ? it.row0 : it.row0 - L.sh_rows;
  const char* hbase = (const char*)(H + (size_t)hrow0 * ld);
  const i32x4 rsW = make_rsrc(wbase, (uint32_t)((int64_t)KT * kStageBytes));
  const i32x4 rsH = make_rsrc(hbase, (uint32_t)((int64_t)it.nrows * ld * 2));

  const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = w >> 1, wn = w & 1;
  uint32_t hoff[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = i * 64 + (tid >> 2);
    const int rr = r < it.nrows ? r : it.nrows - 1;
    hoff[i] = (uint32_t)rr * (uint32_t)(ld * 2) + (uint32_t)(swz_chunk(r, tid & 3) * 16);
  }
  const uint32_t woff = (uint32_t)tid * 16;
  const uint32_t lds_w = lds_offset(lds) + (uint32_t)(w * 1024);

  // stages run over the partitions some row of this tile keeps (Sec. 4: dropped units cost nothing);
  // begin() is called with increasing st, so a running cursor maps st -> K position.
  const int np = sh ? 1 : L.P;
  int nstages = 0;
  for (int p = 0; p < np; ++p) nstages += ((it.kmask >> p) & 1) ? KSp : 0;
  int p_cur = 0, k_in = 0;
  while (p_cur < np && !((it.kmask >> p_cur) & 1)) ++p_cur;
  uint32_t slot = 0, sW = 0, sH = 0;
  auto begin = [&](int st) {
    const int kt = p_cur * KSp + k_in;
    if (++k_in == KSp) {
      k_in = 0;
      ++p_cur;
      while (p_cur < np && !((it.kmask >> p_cur) & 1)) ++p_cur;
    }
    slot = (uint32_t)(st % kStages) * kStagePair + lds_w;
    sH = (uint32_t)(kt * (kBK * 2));
    sW = (uint32_t)(kt * kStageBytes);
  };
  auto one = [&](int q) {
    if (q < 4) dma16(rsH, slot + q * 4096, hoff[q], sH);
    else dma16(rsW, slot + kStageBytes + (q - 4) * 4096, woff, sW + (q - 4) * 4096);
  };

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  mainloop(nstages, begin, one, lds, wm, wn, lane, acc);

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
