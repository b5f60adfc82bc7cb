// bf16 MFMA grouped GEMMs for gfx950 (the hot loops of the layer).
//
//   GEMM-1  H[row][p*Fp + j] = Swish(x_row . W1[:, j]) * (x_row . W3[:, j])   (Eq. 4: gate, up, Swish*mul)
//           one work item = up to 256 rows (token-expert pairs of one expert) x 128 neurons of partition p
//   GEMM-2  Yp[row][d] = sum over the partitions p kept by some row of the tile, sum_j H[row][p*Fp+j] W2[p*Fp+j][d]
//           one work item = up to 256 rows x 256 output columns; dropped partitions are skipped whole
//
// Both kernels: 256 threads = 4 wavefronts, one per SIMD, 256 fp32 accumulator registers each,
// v_mfma_f32_32x32x16_bf16.  A full 256-row tile is split 2 x 2 (each wavefront a 128 x 128 block,
// 4 x 4 MFMA blocks).  The last tile of an expert's (or sub-expert's) row list is ragged: there the
// wavefronts split the weight dimension four ways and all walk the same rows, skipping the
// 32-row blocks past the end, so that a tile with r rows does ceil(r/32)/8 of a full one's matrix
// work (with drops every sub-expert has its own ragged tail: this is what keeps time proportional
// to the kept work); its time does not fall below the arrival of its weight tile, though
// (measured: 0.7 of a full tile for a handful of rows).
// Further variants of GEMM-1: a last neuron tile of at most 64 neurons takes only the first 128
// weight rows, and items of at most 128 rows can be halves of a neuron tile (64 neurons) with a
// ring twice as deep, for batches so small that the kernel only streams weights.
// GEMM-2 feeds the weight fragment as the MFMA's A operand, so that a lane ends up with four
// consecutive output columns of a row.
// The per-pair partial outputs of GEMM-2 (fp32 accumulators) are stored in half precision too unless
// the context asks for fp32 partials: they are the largest stream of the fine-grained layers (K
// partial rows of D values per token, written here and read once by the combine kernel).
// Number formats: GEMM-1 multiplies bf16 by bf16 (x and W1 / W3 as the caller stores them).  The
// intermediate activation H is kept as IEEE half precision (11 significant bits; bf16's 8 cost
// up to 2e-2 of the output RMS on the largest outputs of a batch), so GEMM-2 is the f16 MFMA of
// the same shape and rate, over W2 converted once, exactly, to half precision times a power of
// two by moe_partition_weights.  |H| beyond 65504 saturates.
//
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
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(int)))) int i32x4;

constexpr int kStages = 4;                          // LDS ring depth
constexpr int kStagePair = 2 * kStageBytes;         // A tile + B tile of one stage: 32 KiB
constexpr int kLdsBytes = kStages * (kStagePair + 64 * kBK * 2);  // 144 KiB: four stages of the tallest tile (16 KiB A + 320 rows of B)
// An LDS ring: NS stages, SB bytes apart, the MFMA B tile BOFF bytes into a stage.
template <int NS_, int SB_, int BOFF_>
struct Ring {
  static constexpr int NS = NS_, SB = SB_, BOFF = BOFF_, BYTES = NS_ * SB_;
};
using RingWhole = Ring<kStages, kStagePair, kStageBytes>;  // 16 KiB A tile + 16 KiB B tile
// half-tile items of GEMM-1 (at most 128 rows): 8 KiB of weights + 8 KiB of rows, twice as deep
using RingHalf = Ring<8, kStageBytes, kStageBytes / 2>;
static_assert(RingHalf::BYTES <= kLdsBytes, "same allocation");
// tall tiles of GEMM-1 (a full row tile that also takes the expert's last 1..64 rows): 16 KiB A tile + 320 rows of B
constexpr int kTallRows = kMfmaBM + 64;
using RingTall = Ring<kStages, kStageBytes + kTallRows * (kBK * 2), kStageBytes>;
static_assert(RingTall::BYTES <= kLdsBytes, "same allocation");
// the same for GEMM-2, whose A tile holds the rows: 320 rows of A + 16 KiB B tile
using RingTall2 = Ring<kStages, kStageBytes + kTallRows * (kBK * 2), kTallRows * (kBK * 2)>;
constexpr int64_t kStreamOutBytes = 192ll << 20;    // GEMM-2 outputs larger than this bypass the caches (256 MiB of last-level cache, shared with H)
constexpr int kLoadsPerStage = 2 * (kStageBytes / 16 / 256);  // per thread: 4 (A) + 4 (B)
constexpr uint32_t kRsrcFlags = 0x00020000u;        // raw buffer, 32-bit elements
constexpr int kRowBytes = kBK * 2;                  // one tile row in LDS: 64 bytes
constexpr float kHalfMax = 65504.f;                 // largest finite half-precision value

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

// This thread's index in the workgroup, worked out anew from the wavefront's index (a scalar) and the lane id.
// The tile functions below start from it instead of from a value handed down: a thread index that lives
// in one register from the top of the kernel through all of its variants is what the register allocator
// parks in scratch first (volatile, so that the copies are not merged back into one).
__device__ __forceinline__ int fresh_tid(int w) {
  int lane;
  asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(lane));
  return (w << 6) | lane;
}

// XCD-aware order: consecutive block ids land on different XCDs (round robin over 8), so give
// each XCD a run of 32 consecutive work items out of every 256: items that share a weight tile
// then share an L2.
__device__ __forceinline__ int xcd_remap(int b) {
  const int chunk = b >> 8, within = b & 255;
  return (chunk << 8) + ((within & 7) << 5) + (within >> 3);
}

// Operand fragments of one K substep (16 values of K): I blocks of 32 A rows, J blocks of 32 B rows.
template <int I, int J>
struct Frags {
  bf16x8 a[I], b[J];
  bf16x8 bx;  // tall tiles: one more block of B rows
};

// One wavefront's share of the tile product.
//   I x J   MFMA blocks (32 x 32) of this wavefront; I * J == 16, or 8 for a tile of half the weight rows.
//   NI / NJ: only the first NI (NJ) blocks of that dimension hold rows (ragged tile); the others
//   are neither read nor multiplied.  They are template parameters, not run-time values: branches
//   around single MFMAs would push the accumulators out of their registers.
// The main loop below is shared by both GEMMs:
//   begin(st): fix the ring slot and the K offsets of stage st (called once per stage, in order);
//   one(q):    enqueue this thread's q-th DMA load (0..NLOADS-1) of the stage begun last: first the
//              loads of the weight tile (4; 2 for half a tile), then one per 64 pair rows that exist.
// On return every DMA has completed and acc holds the tile.
//
// Per stage a wavefront issues 32 MFMAs (1024 matrix-core cycles; half of that when I * J == 8),
// I+J LDS reads per substep and up to 8 DMA loads.  With one wavefront per SIMD nothing else hides
// an instruction that stalls the stream, so the reads and loads are threaded between the MFMAs by
// hand and pinned with scheduling barriers.
// F16: the operands are half precision (GEMM-2) instead of bf16; the fragments are 16 bytes either way.
// EX (tall tiles): the wavefront also multiplies its four weight blocks (the A blocks of GEMM-1, the B blocks
// of GEMM-2) with one more block of 32 pair rows (bx).  The 256 accumulation registers are taken, so these
// products accumulate in ordinary registers, which the compiler only allows for all matrix instructions of a
// kernel or none: they are written as inline assembly.  Nothing but the next such instruction (and, much
// later, the epilogue) touches their registers.
template <int I, int J, int NI, int NJ, int NLOADS, bool SWAP = false, int NS = kStages, int SB = kStagePair, int BOFF = kStageBytes,
          bool F16 = false, bool EX = false>
struct WaveTile {
  static_assert(I * J == 16 || I * J == 8, "256 or 128 accumulator registers");
  static_assert(!EX || (I == 4 && J == 4 && NI == I && NJ == J && SWAP == F16), "extra block: full tiles of GEMM-1 (bf16) or GEMM-2 (f16, operands swapped)");
  static constexpr int M = I * J;  // MFMAs per K substep
  static_assert(NLOADS >= 1 && NLOADS <= kLoadsPerStage + (EX ? 1 : 0), "DMA loads per thread and stage");
  f32x16 acc[I][J];
  f32x16 accx[EX ? 4 : 1];  // EX: weight block k x the extra block of pair rows
  uint32_t offA, offB;  // byte offset of this lane's row in the A / B tile of a stage (block 0)
  uint32_t offBx;       // EX: the same for the extra block of pair rows (in the B tile of GEMM-1, the A tile of GEMM-2)
  int bx_mode;          // EX, the same for the whole wavefront: 0 no extra block; 3: all four weight blocks x the extra block;
                        // 1: only the first two (the wavefront that shares the weight blocks takes the other two)
  uint32_t offW2;       // EX: byte offset of weight blocks 2 and 3.  Weight fragment k is block (k + rot) & 3 of the wavefront's
                        // four: with rot = 2 the wavefront's "first two" blocks are the other wavefront's last two
  uint32_t c0, c1;      // swizzled chunk offset of substep 0 / 1

  // bx_row0: first row of the extra block of pair rows (mode != 0); rot: see offW2
  __device__ __forceinline__ void init(int a_row0, int b_row0, int lane, int bx_row0 = 0, int mode = 0, int rot = 0) {
    bx_mode = EX ? mode : 0;
    offBx = (uint32_t)(bx_row0 + (lane & 31)) * kRowBytes + (SWAP ? 0 : BOFF);
    if (EX) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) accx[i][v] = 0.f;
    }
    const int r32 = lane & 31, half = lane >> 5;
    const int sw = (r32 >> 2) & 3;
    offA = (uint32_t)(a_row0 + r32) * kRowBytes;
    offB = (uint32_t)(b_row0 + r32) * kRowBytes + BOFF;
    // weight fragments 2, 3 sit at offW2 + (k - 2) * 2 KiB, fragments 0, 1 at the (rotated) block offset + k * 2 KiB
    offW2 = (SWAP ? offB : offA) + (uint32_t)(((2 + rot) & 3) * 32 * kRowBytes);
    if (EX) (SWAP ? offB : offA) += (uint32_t)(rot * 32 * kRowBytes);
    c0 = (uint32_t)((half ^ sw) * 16);
    c1 = (uint32_t)(((2 + half) ^ sw) * 16);
#pragma unroll
    for (int i = 0; i < I; ++i)
#pragma unroll
      for (int j = 0; j < J; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  }

  static constexpr __device__ __forceinline__ bool act_i(int i) { return i < NI; }
  static constexpr __device__ __forceinline__ bool act_j(int j) { return j < NJ; }

  // k-th fragment read of a substep, in the order the MFMA sequence first needs them:
  // a0, b0 .. b(J-1), a1 .. a(I-1)
  __device__ __forceinline__ void read_k(Frags<I, J>& f, const char* stage, uint32_t c, int k) const {
    if (k == 0) {
      f.a[0] = *(const bf16x8*)(stage + offA + c);
    } else if (k <= J) {
      const int j = k - 1;
      if (act_j(j)) f.b[j] = *(const bf16x8*)(stage + (EX && SWAP && j >= 2 ? offW2 + (j - 2) * (32 * kRowBytes) : offB + j * (32 * kRowBytes)) + c);
    } else if (k < I + J) {
      const int i = k - J;
      if (act_i(i)) f.a[i] = *(const bf16x8*)(stage + (EX && !SWAP && i >= 2 ? offW2 + (i - 2) * (32 * kRowBytes) : offA + i * (32 * kRowBytes)) + c);
    } else if (EX) {
      if (bx_mode) f.bx = *(const bf16x8*)(stage + offBx + c);
    }
  }

  __device__ __forceinline__ void read_all(Frags<I, J>& f, const char* stage, uint32_t c) const {
#pragma unroll
    for (int k = 0; k < I + J + (EX ? 1 : 0); ++k) read_k(f, stage, c, k);
  }

  // 16 MFMAs on `cur`; between them the I+J reads of the next substep into `nxt` and, if DMA,
  // the 8 loads of a later stage.
  template <bool READS, bool DMA, class One>
  __device__ __forceinline__ void half_stage(const Frags<I, J>& cur, Frags<I, J>& nxt, const char* nxt_stage, uint32_t nxt_c,
                                            One&& one) {
    constexpr int R = I + J + (EX ? 1 : 0);
#pragma unroll
    for (int m = 0; m < M; ++m) {
      const int i = m / J, j = m % J;
      if (act_i(i) && act_j(j)) {
        const bf16x8 fa = SWAP ? cur.b[j] : cur.a[i], fb = SWAP ? cur.a[i] : cur.b[j];
        if (F16)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, fa), __builtin_bit_cast(f16x8, fb), acc[i][j], 0, 0, 0);
        else
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc[i][j], 0, 0, 0);
      }
      if (M == 16) {  // a DMA slot after every second MFMA, or after every one of 8
        if (DMA && (m & 1) && (m >> 1) < NLOADS) one(m >> 1);
        if (DMA && m == 0 && NLOADS > 8) one(8);  // the ninth load of a tall tile
      } else {
        if (DMA && m < NLOADS) one(m);
      }
      if (READS) {
#pragma unroll
        for (int k = (m * R) / M; k < ((m + 1) * R) / M; ++k) read_k(nxt, nxt_stage, nxt_c, k);
      }
      if (m & 1) __builtin_amdgcn_sched_barrier(0);
    }
    // the extra block's products last: their operands have long arrived (first, they would wait for the
    // LDS reads issued at the end of the half stage before)
    if constexpr (EX) {
      // the weight fragment is the MFMA's first operand in both GEMMs (a[k] of GEMM-1, b[k] of GEMM-2)
#define DSMOE_EXTRA_MFMA(K)                                                                                                      \
  if (F16) asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+v"(accx[K]) : "v"(cur.b[K]), "v"(cur.bx));                \
  else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(accx[K]) : "v"(cur.a[K]), "v"(cur.bx))
      DSMOE_EXTRA_MFMA(0);
      DSMOE_EXTRA_MFMA(1);
      if (bx_mode == 3) {
        DSMOE_EXTRA_MFMA(2);
        DSMOE_EXTRA_MFMA(3);
      }
#undef DSMOE_EXTRA_MFMA
    }
  }

  // s_waitcnt takes an immediate: all but the last k stages' loads of this thread have landed
  static __device__ __forceinline__ void wait_stages(int k) {
    static_assert((NS - 2) * NLOADS < 64, "vmcnt is a 6-bit counter");
    switch (k) {
      case 0: wait_vm<0>(); break;
      case 1: wait_vm<NLOADS>(); break;
      case 2: wait_vm<(NS > 3 ? 2 : 0) * NLOADS>(); break;
      case 3: wait_vm<(NS > 4 ? 3 : 0) * NLOADS>(); break;
      case 4: wait_vm<(NS > 5 ? 4 : 0) * NLOADS>(); break;
      case 5: wait_vm<(NS > 6 ? 5 : 0) * NLOADS>(); break;
      default: wait_vm<(NS > 7 ? 6 : 0) * NLOADS>(); break;
    }
  }

  // Ring of NS stages, SB bytes apart; stage st + NS - 1 is enqueued while stage st is multiplied.
  template <class Begin, class One>
  __device__ __forceinline__ void mainloop(int n, Begin&& begin, One&& one, const char* lds) {
    static_assert(NS >= 3 && NS <= 8, "ring depth");
    constexpr int PD = NS - 1;  // prefetch distance
    Frags<I, J> f0, f1;
    if (n <= 0) return;
    auto issue_all = [&](int st) {
      begin(st);
#pragma unroll
      for (int q = 0; q < NLOADS; ++q) one(q);
    };
#pragma unroll
    for (int s = 0; s < PD; ++s)
      if (s < n) issue_all(s);
    wait_stages((n < PD ? n : PD) - 1);
    block_barrier();
    read_all(f0, lds, c0);
    // c1 is first needed inside the loop; if the register allocator parked it in scratch, make it
    // come back (and be waited for) here, so that no s_waitcnt vmcnt(0) lands inside the loop
    // and drains the DMA queue every iteration
    asm volatile("" ::"v"(c1), "v"(offA), "v"(offB));
    int st = 0;
    for (; st + PD < n; ++st) {
      const char* cur = lds + (st % NS) * SB;
      // first half: multiply substep 0 while the substep 1 operands stream in from LDS
      half_stage<true, false>(f0, f1, cur, c1, one);
      // stage st+1 must have landed for every wave (the later ones may still be in flight); after
      // the barrier every wave has also finished reading stage st-1, whose slot stage st+PD takes
      wait_vm<(PD - 2) * NLOADS>();
      block_barrier();
      begin(st + PD);
      // second half: multiply substep 1; between the MFMAs enqueue stage st+PD and fetch substep 0 of stage st+1
      const char* nxt = lds + ((st + 1) % NS) * SB;
      half_stage<true, true>(f1, f0, nxt, c0, one);
    }
    for (; st + 1 < n; ++st) {  // last stages: nothing left to enqueue
      const char* cur = lds + (st % NS) * SB;
      half_stage<true, false>(f0, f1, cur, c1, one);
      wait_stages(n - 2 - st);
      block_barrier();
      const char* nxt = lds + ((st + 1) % NS) * SB;
      half_stage<true, false>(f1, f0, nxt, c0, one);
    }
    const char* last = lds + ((n - 1) % NS) * SB;
    half_stage<true, false>(f0, f1, last, c1, one);
    half_stage<false, false>(f1, f0, last, c0, one);
  }
};

// ------------------------------------------------------------------------------------- GEMM-1
struct G1Args {
  Item1 it;
  bool sh;
  int KS1, Fp, ld, hrow0, epi;
  i32x4 rsW, rsX;
  uint32_t lds_w;
  const int32_t* row_token;  // token of every pair row
  uint32_t x_row_bytes;
  const uint8_t* row_bits;
  uint16_t* H;
};

// MFMA A = weight rows, B = pair rows.  Weight rows come in blocks of 32: block 2b is the gate
// projection of neurons 32b .. 32b+31 of the tile, block 2b+1 their up projection.
// NW / NX: 4 KiB loads per thread and stage for the weight tile / for the rows (64 rows each).
// TALL: a full row tile that also takes the 1..64 rows its expert has beyond it (rows 256..319 of the item: each
// wavefront multiplies its four weight blocks with one more block of 32 rows, see WaveTile), so that those
// rows do not pull the whole weight tile through a second compute unit.
template <int I, int J, int NJ, bool PROFILE, int NW = 4, bool HALF = false, class RING = RingWhole, int NX = (J == 8 ? (NJ * 32 + 63) / 64 : 4),
          bool TALL = false>
__device__ __forceinline__ void gemm1_tile(const G1Args& g, char* lds, int a_row0, int b_row0, int w) {
  static_assert(!TALL || (I == 4 && J == 4 && NJ == 4 && NW == 4 && !HALF && NX == 5 && !PROFILE), "tall tiles: 2 x 2 wavefronts, 320 rows, the layer's pass only");
  // Each instantiation derives its lane-dependent offsets from its own copy of the thread id:
  // shared, they would stay live across all the instantiations of the kernel and be parked in
  // scratch, and a scratch reload inside a main loop waits for vmcnt(0), which drains the DMA queue.
  int tid = fresh_tid(w);
  const int lane = tid & 63;
  // the ragged layout (J == 8) walks all pair rows: only the 64-row groups that exist are loaded
  // HALF: one half (64 neurons) of a neuron tile under at most 128 pair rows, in the streaming
  // regime: stages of 8 KiB of weights + 8 KiB of rows in a ring of 8, so that as many bytes are in
  // flight as with whole tiles; wavefronts 2 and 3 only help to load (NJ == 0).
  constexpr int NS = RING::NS, SB = RING::SB, BOFF = RING::BOFF;
  const int half = HALF ? g.it.half - 1 : 0;
  WaveTile<I, J, I, NJ, NW + NX, false, NS, SB, BOFF, false, TALL> t;
  // tall tiles, up to 32 extra rows: both wavefronts of a weight half take rows 256..287, two weight blocks each;
  // up to 64: the wavefronts of the first / second half of the rows take rows 256..287 / 288..319, all four blocks
  const bool two_blocks = g.it.nrows > kMfmaBM + 32;
  const int bx_row0 = kMfmaBM + (two_blocks ? b_row0 >> 2 : 0);
  const int arot = TALL && !two_blocks && b_row0 ? 2 : 0;  // which two of the four weight blocks are this wavefront's "first two"
  t.init(a_row0, b_row0, lane, bx_row0, !TALL ? 0 : two_blocks ? 3 : 1, arot);
  // this thread's part of the activation gather: chunk (tid & 3) of rows i * 64 + (tid >> 2).  Worked out
  // here, per instantiation, for the same reason as the lane offsets above.
  uint32_t xoff[NX];
#pragma unroll
  for (int i = 0; i < NX; ++i) {
    const int r = i * 64 + (tid >> 2);
    const int rr = r < g.it.nrows ? r : g.it.nrows - 1;  // rows past the end re-read the last valid row
    xoff[i] = (uint32_t)g.row_token[g.it.row0 + rr] * g.x_row_bytes + (uint32_t)(swz_chunk(r, tid & 3) * 16);
  }
  const uint32_t woff = (uint32_t)tid * 16;  // the weight tile is a linear stream: 16 bytes per thread and 4 KiB slab
  uint32_t slot = 0, sW = 0, sX = 0;
  auto begin = [&](int st) {
    slot = (uint32_t)(st % NS) * SB + g.lds_w;
    sW = (uint32_t)(st * kStageBytes + half * (kStageBytes / 2));
    sX = (uint32_t)(st * kRowBytes);
  };
  auto one = [&](int q) {
    if (q < NW) dma16(g.rsW, slot + q * 4096, woff, sW + q * 4096);
    else dma16(g.rsX, slot + BOFF + (q - NW) * 4096, xoff[q - NW], sX);
  };
  t.mainloop(g.KS1, begin, one, lds);
  // the epilogue's addresses hang on a fresh copy of the thread id: worked out before the main
  // loop (where the compiler would move them) they would occupy registers all the way through it
  tid = fresh_tid(w);
  const int le = tid & 63;

  if constexpr (PROFILE) {
    // Importance profiling (Sec. 4.2 b): the metric of every (row, neuron) of the tile is summed over
    // the rows right here, in fp32: over the wavefront's row blocks in registers, over the 32 lanes
    // that hold different rows of the same neurons by a fixed exchange pattern, over the two
    // wavefronts that split the rows through LDS.  The tile's 128 sums go to row (row tile) of a
    // [row tiles][F] table that colsum_tiles_kernel adds up per expert, in tile order.  Nothing is
    // rounded to 16 bits and no per-row intermediate is written.
    float* part = (float*)lds;  // [2 row groups][128 neurons]
    const bool with_up = g.epi >= 3, magnitude = g.epi == 2 || g.epi == 4;  // the four metrics, see epi_value
    block_barrier();            // every wave is done reading the last stage
    if (tid < 256) part[tid] = 0.f;
    uint32_t keptmask = 0;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int r = b_row0 + j * 32 + (le & 31);
      const bool kept = r < g.it.nrows && ((g.row_bits[g.it.row0 + (r < g.it.nrows ? r : 0)] >> g.it.p) & 1);
      keptmask |= (kept ? 1u : 0u) << j;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < I; i += 2) {
      float sum[16];
#pragma unroll
      for (int v = 0; v < 16; ++v) sum[v] = 0.f;
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const bool kept = (keptmask >> j) & 1;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float sg = silu_fast(t.acc[i][j][v]);
          float m = with_up ? sg * t.acc[i + 1][j][v] : sg;  // uniform selects, no branch per value
          m = magnitude ? fabsf(m) : m;
          sum[v] += kept ? m : 0.f;
        }
      }
      if (NJ > 0) {
        const int nb = (a_row0 >> 5) + i + 4 * half;  // weight block index; neurons of the tile: (nb/2)*32 ..
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          float x = row_sum(sum[v]);   // over the sixteen lanes of a row, then the two rows of this half of the wavefront
          x += __shfl_xor(x, 16, 64);  // (a + b in one lane, b + a in the other: the same bits)
          if ((le & 31) == 0) part[(b_row0 ? 128 : 0) + (nb >> 1) * 32 + 8 * (v >> 2) + 4 * (le >> 5) + (v & 3)] = x;
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    __syncthreads();
    const int n_lo = HALF ? 64 * half : 0, n_hi = HALF ? n_lo + 64 : kMfmaNeur;
    if (tid >= n_lo && tid < n_hi && g.it.jt * kMfmaNeur + tid < g.Fp) {
      float* table = (float*)g.H;  // the profiling pass keeps its per-tile sums where the layer keeps H
      const size_t tile = (size_t)(g.hrow0 / kMfmaBM);
      table[tile * g.ld + (size_t)g.it.p * g.Fp + g.it.jt * kMfmaNeur + tid] = part[tid] + part[128 + tid];
    }
    return;
  }

  // epilogue.  acc[i][j][v]: weight row a_row0 + i*32 + 8*(v/4) + 4*(lane/32) + v%4, pair row
  // b_row0 + j*32 + lane%32.  Swish(gate) * up is rounded to half precision and parked in LDS as a
  // [256 rows][128 neurons] tile (320 rows in a tall tile; rows padded to 272 bytes against bank conflicts), then written
  // out in whole 256-byte row segments: 16 lanes per row, 16 bytes per lane.
  constexpr int kHsRow = kMfmaNeur * 2 + 16;
  block_barrier();  // every wave is done reading the last stage
  // one block of 32 rows x 32 neurons: gate and up accumulators of weight blocks i and i + 1, pair row r of this lane
  auto emit = [&](const f32x16& gate, const f32x16& up, int r, bool kept, int i) {
    const int nb = (a_row0 >> 5) + ((i + arot) & 3) + 4 * half;  // weight block index; neurons of the tile: (nb/2)*32 ..
    char* srow = lds + r * kHsRow + ((nb >> 1) * 32 + (le >> 5) * 4) * 2;
    // one branch per block of sixteen values, so that their chains of dependent operations interleave
    // (a select per value makes the compiler branch around every single evaluation)
    if (kept) {
#pragma unroll
      for (int vq = 0; vq < 4; ++vq) {
        float h[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) h[c] = epi_value<true>(0, gate[vq * 4 + c], up[vq * 4 + c]);  // Swish(gate) * up (Eq. 4)
        // half precision, round to nearest: half a unit of the kept 10 fraction bits is added to the
        // magnitude (fp32 bit pattern + 2^12), then the packed conversion truncates.  Truncation never
        // yields infinity, so |h| beyond 65504 saturates.
#pragma unroll
        for (int c = 0; c < 4; ++c) h[c] = __uint_as_float(__float_as_uint(h[c]) + 0x1000u);
        uint2 pk;
        pk.x = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(h[0], h[1]));
        pk.y = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(h[2], h[3]));
        *(uint2*)(srow + vq * 16) = pk;
      }
    } else {
#pragma unroll
      for (int vq = 0; vq < 4; ++vq) *(uint2*)(srow + vq * 16) = make_uint2(0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);  // one block of rows and 32 neurons at a time: keeps the register pressure of the epilogue low
  };
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int r = b_row0 + j * 32 + (le & 31);
    const bool kept = r < g.it.nrows && ((g.row_bits[g.it.row0 + (r < g.it.nrows ? r : 0)] >> g.it.p) & 1);
#pragma unroll
    for (int i = 0; i < I; i += 2) emit(t.acc[i][j], t.acc[i + 1][j], r, kept, i);
  }
  if constexpr (TALL) {
    const int r = bx_row0 + (le & 31);
    const bool kept = r < g.it.nrows && ((g.row_bits[g.it.row0 + (r < g.it.nrows ? r : 0)] >> g.it.p) & 1);
    emit(t.accx[0], t.accx[1], r, kept, 0);
    if (t.bx_mode == 3) emit(t.accx[2], t.accx[3], r, kept, 2);
  }
  __syncthreads();
  const int n_in = g.it.jt * kMfmaNeur + (tid & 15) * 8;  // first of this lane's 8 neurons, inside the partition
  if (n_in < g.Fp && (!HALF || ((tid & 15) >> 3) == half)) {
    // four rows at a time: their reads first, whether or not the rows exist (pinned here: inside the
    // branch each read would wait for its own LDS round trip), then the stores
    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
#pragma unroll 1
    for (int c0 = 0; c0 < kTallRows / 16; c0 += 4) {  // up to 320 rows: the tile before an expert's short last tile zero-fills that one's rows too
      u32x4_t v[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) v[c] = *(const u32x4_t*)(lds + ((c0 + c) * 16 + (tid >> 4)) * kHsRow + (tid & 15) * 16);
#pragma unroll
      for (int c = 0; c < 4; ++c) asm volatile("" : "+v"(v[c]));
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int r = (c0 + c) * 16 + (tid >> 4);
        if (r < g.it.nfill)  // rows [nrows, nfill) of the row tile keep nothing of this partition: zeros
          *(u32x4_t*)(g.H + (size_t)(g.hrow0 + r) * g.ld + (size_t)g.it.p * g.Fp + n_in) = r < g.it.nrows ? v[c] : u32x4_t{0, 0, 0, 0};
      }
    }
  }
}

// What every GEMM-1 workgroup does first: its item and the buffer descriptors.
__device__ __forceinline__ void gemm1_setup(G1Args& g, int item_id, const Layout& L, int T, const char* packed, const uint16_t* x, char* ws,
                                            int epi, const char* lds, int tid, int w) {
  g.it = ((const Item1*)(ws + L.o_items1))[item_id];
  g.row_bits = (const uint8_t*)(ws + L.o_row_bits);
  g.row_token = (const int32_t*)(ws + L.o_row_token);
  g.x_row_bytes = (uint32_t)(L.D * 2);
  g.sh = g.it.e == L.E_res;
  g.KS1 = L.D / kBK;
  g.Fp = g.sh ? L.F_shT : L.Fp;
  g.ld = g.sh ? L.F_shT : L.F;
  const char* wbase = g.sh ? packed + L.p_sw13 + (int64_t)g.it.jt * g.KS1 * kStageBytes
                           : packed + L.p_w13 + (((int64_t)g.it.e * L.P + g.it.p) * L.NT1 + g.it.jt) * g.KS1 * kStageBytes;
  g.rsW = make_rsrc(wbase, (uint32_t)(g.KS1 * kStageBytes));
  g.rsX = make_rsrc(x, (uint32_t)((int64_t)T * L.D * 2));
  g.H = g.sh ? (uint16_t*)(ws + L.o_Hs) : (uint16_t*)(ws + L.o_H);
  g.hrow0 = g.sh ? g.it.row0 : g.it.row0 - L.sh_rows;
  g.epi = epi;

  g.lds_w = lds_offset(lds) + (uint32_t)(w * 1024);  // this wavefront's 1 KiB slice of each 4 KiB slab
}

// PROFILE = false is the layer's kernel: it stores Swish(gate) * up.  PROFILE = true is the importance
// profiling pass: it picks the metric at run time (epi 1..4), sums it over the rows of the tile and
// stores 128 column sums per item instead of the activation.
template <bool PROFILE>
__global__ __launch_bounds__(256) void gemm1_mfma_kernel(Layout L, int T, const char* packed, const uint16_t* x, char* ws, int epi) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int item_id = xcd_remap(blockIdx.x);
  if (item_id >= ((const int32_t*)(ws + L.o_counters))[0]) return;  // past the end of the list
  const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid >> 6);
  G1Args g;
  gemm1_setup(g, item_id, L, T, packed, x, ws, epi, lds, tid, w);
  if (PROFILE && g.sh) return;  // importance is profiled for the routed experts only

  if (g.it.half) {  // at most 128 rows (the plan guarantees it): wavefronts 0 and 1 multiply, 64 weight rows each
    if (w < 2) {
      switch ((g.it.nrows + 31) >> 5) {
        case 1: gemm1_tile<2, 4, 1, PROFILE, 2, true, RingHalf, 2>(g, lds, w * 64, 0, w); break;
        case 2: gemm1_tile<2, 4, 2, PROFILE, 2, true, RingHalf, 2>(g, lds, w * 64, 0, w); break;
        case 3: gemm1_tile<2, 4, 3, PROFILE, 2, true, RingHalf, 2>(g, lds, w * 64, 0, w); break;
        default: gemm1_tile<2, 4, 4, PROFILE, 2, true, RingHalf, 2>(g, lds, w * 64, 0, w); break;
      }
    } else {
      gemm1_tile<2, 4, 0, PROFILE, 2, true, RingHalf, 2>(g, lds, 0, 0, w);
    }
  } else if (!PROFILE && g.it.nrows > kMfmaBM) {  // a full row tile and the expert's last 1..64 rows (the profiling pass plans without them)
    gemm1_tile<4, 4, 4, false, 4, false, RingTall, 5, true>(g, lds, (w >> 1) * 128, (w & 1) * 128, w);
  } else if (g.it.nrows == kMfmaBM) {
    // 2 x 2 wavefronts, 128 weight rows x 128 pair rows each; a last neuron tile that is at most half
    // full takes the first 128 weight rows only (64 x 128 per wavefront)
    if (g.Fp - g.it.jt * kMfmaNeur <= kMfmaNeur / 2) gemm1_tile<2, 4, 4, PROFILE, 2>(g, lds, (w >> 1) * 64, (w & 1) * 128, w);
    else gemm1_tile<4, 4, 4, PROFILE>(g, lds, (w >> 1) * 128, (w & 1) * 128, w);
  } else {  // 4 x 1: 64 weight rows x the ceil(nrows/32) blocks of pair rows that exist
    switch ((g.it.nrows + 31) >> 5) {
      case 1: gemm1_tile<2, 8, 1, PROFILE>(g, lds, w * 64, 0, w); break;
      case 2: gemm1_tile<2, 8, 2, PROFILE>(g, lds, w * 64, 0, w); break;
      case 3: gemm1_tile<2, 8, 3, PROFILE>(g, lds, w * 64, 0, w); break;
      case 4: gemm1_tile<2, 8, 4, PROFILE>(g, lds, w * 64, 0, w); break;
      case 5: gemm1_tile<2, 8, 5, PROFILE>(g, lds, w * 64, 0, w); break;
      case 6: gemm1_tile<2, 8, 6, PROFILE>(g, lds, w * 64, 0, w); break;
      case 7: gemm1_tile<2, 8, 7, PROFILE>(g, lds, w * 64, 0, w); break;
      default: gemm1_tile<2, 8, 8, PROFILE>(g, lds, w * 64, 0, w); break;
    }
  }
}

// ------------------------------------------------------------------------------------- GEMM-2
struct G2Args {
  Item2 it;
  int np, KSp, nstages, D;
  i32x4 rsW, rsH;
  uint32_t lds_w, h_row_bytes;
  char* Y;       // where row 0, column 0 of this item's output tile goes (float, or half precision: YH)
  int ldy;       // its row stride in elements: D in Yp, 256 in a pool tile
  float yscale;  // YH: the accumulators are stored times this power of two (see kYpHalfScale)
};

// MFMA A = pair rows of H, B = output columns of W2 (both half precision).
// YH: the partial outputs are stored in half precision (see launch_gemm2_mfma)
// TALL: a full row tile that also takes the 1..64 rows of its expert's short last tile (see gemm1_tile): rows
// 256..319 of the item, one more block of 32 rows per wavefront, times all four of its column blocks or, when
// there is only one such block, times two of them (the wavefront that shares the columns takes the other two).
template <int I, int J, int NI, bool NT, bool YH, class RING = RingWhole, bool TALL = false>
__device__ __forceinline__ void gemm2_tile(const G2Args& g, char* lds, int a_row0, int b_row0, int w) {
  static_assert(!TALL || (I == 4 && J == 4 && NI == 4), "tall tiles: 2 x 2 wavefronts, 320 rows");
  int tid = fresh_tid(w);  // see gemm1_tile
  const int lane = tid & 63;
  constexpr int NH = TALL ? 5 : I == 8 ? (NI * 32 + 63) / 64 : 4;  // loads per thread and stage for the rows of H (64 rows each)
  WaveTile<I, J, NI, J, 4 + NH, true, RING::NS, RING::SB, RING::BOFF, true, TALL> t;
  const bool two_blocks = g.it.nrows > kMfmaBM + 32;
  const int bx_row0 = kMfmaBM + (two_blocks ? a_row0 >> 2 : 0);
  const int rot = TALL && !two_blocks && a_row0 ? 2 : 0;  // column block of accumulator j: (j + rot) & 3
  t.init(a_row0, b_row0, lane, bx_row0, !TALL ? 0 : two_blocks ? 3 : 1, rot);
  // this thread's part of the rows of H: chunk (tid & 3) of rows i * 64 + (tid >> 2) (per instantiation, see gemm1_tile)
  uint32_t hoff[NH];
#pragma unroll
  for (int i = 0; i < NH; ++i) {
    const int r = i * 64 + (tid >> 2);
    const int rr = r < g.it.nrows ? r : g.it.nrows - 1;
    hoff[i] = (uint32_t)rr * g.h_row_bytes + (uint32_t)(swz_chunk(r, tid & 3) * 16);
  }
  // stages run over the partitions some row of this tile keeps (Sec. 4: dropped units cost nothing);
  // begin() is called with increasing st, so a running cursor maps st -> K position.
  int p_cur = 0, k_in = 0;
  while (p_cur < g.np && !((g.it.kmask >> p_cur) & 1)) ++p_cur;
  const uint32_t woff = (uint32_t)tid * 16;
  uint32_t slot = 0, sW = 0, sH = 0;
  auto begin = [&](int st) {
    const int kt = p_cur * g.KSp + g.it.ks_lo + k_in;
    if (++k_in == g.it.ks_n) {
      k_in = 0;
      ++p_cur;
      while (p_cur < g.np && !((g.it.kmask >> p_cur) & 1)) ++p_cur;
    }
    slot = (uint32_t)(st % RING::NS) * RING::SB + g.lds_w;
    sH = (uint32_t)(kt * kRowBytes);
    sW = (uint32_t)(kt * kStageBytes);
  };
  auto one = [&](int q) {
    if (q < 4) dma16(g.rsW, slot + RING::BOFF + q * 4096, woff, sW + q * 4096);
    else dma16(g.rsH, slot + (q - 4) * 4096, hoff[q - 4], sH);
  };
  t.mainloop(g.nstages, begin, one, lds);
  tid = fresh_tid(w);  // see gemm1_tile: the epilogue's addresses are worked out after the main loop
  const int le = tid & 63;

  // epilogue.  The weight fragment is the MFMA's A operand, so acc[i][j][v] is pair row
  // a_row0 + i*32 + lane%32, column b_row0 + j*32 + 8*(v/4) + 4*(lane/32) + v%4.  Each wavefront
  // turns one block of 32 rows at a time around in its own quarter of the (now idle) ring and
  // writes it out as whole row segments of J*128 bytes, 16 bytes per lane.
  typedef float f32x4_t __attribute__((ext_vector_type(4)));
  constexpr int kEl = YH ? 2 : 4;                // bytes of one stored value
  constexpr int kYsRow = J * 32 * kEl + 16;      // bytes; the pad spreads the rows over the banks
  constexpr int kLanesRow = J * 2 * kEl;         // lanes that share a row in the write-out (16 bytes each)
  constexpr int kColsLane = 16 / kEl;            // columns a lane writes out
  constexpr int kRowsPass = 64 / kLanesRow;      // rows per store instruction
  char* mine = lds + w * (RING::BYTES / 4);
  static_assert(32 * kYsRow <= RING::BYTES / 4, "a block of 32 rows fits a wavefront's quarter of the ring");
  block_barrier();  // every wave is done reading the last stage
  const int cw = g.it.jd * kMfmaBN2 + b_row0 + (le % kLanesRow) * kColsLane;  // first of this lane's columns in the write-out
  // one block of 32 rows: accumulators A[0..nj) (column block (j + rot) & 3 each), first row row_blk of the item
  auto out_block = [&](const f32x16* A, int nj, int row_blk) {
#pragma unroll
    for (int j = 0; j < J; ++j) {
      if (j >= nj) continue;
      const int jc = TALL ? (j + rot) & 3 : j;
#pragma unroll
      for (int vq = 0; vq < 4; ++vq) {
        char* at = mine + (le & 31) * kYsRow + (jc * 32 + vq * 8 + (le >> 5) * 4) * kEl;
        if constexpr (YH) {  // times 2^-10, saturating, round to nearest even
          float v[4];
#pragma unroll
          for (int c = 0; c < 4; ++c) v[c] = __builtin_amdgcn_fmed3f(A[j][vq * 4 + c] * g.yscale, -kHalfMax, kHalfMax);
          f16x2 lo, hi;
          lo[0] = (_Float16)v[0], lo[1] = (_Float16)v[1], hi[0] = (_Float16)v[2], hi[1] = (_Float16)v[3];
          uint2 pk;
          pk.x = __builtin_bit_cast(uint32_t, lo);
          pk.y = __builtin_bit_cast(uint32_t, hi);
          *(uint2*)at = pk;
        } else {
          f32x4_t o;
          o.x = A[j][vq * 4 + 0];
          o.y = A[j][vq * 4 + 1];
          o.z = A[j][vq * 4 + 2];
          o.w = A[j][vq * 4 + 3];
          *(f32x4_t*)at = o;
        }
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // this lane's columns of the write-out belong to column block (first column / 32): written above?
    const bool cols_here = nj == J || ((((le % kLanesRow) * kColsLane >> 5) - rot) & 3) < nj;
    // the reads of up to four passes first, whether or not the row exists (they are pinned here: inside the
    // branches below each would wait for its own LDS round trip), then the stores of the rows that do
    constexpr int kPasses = 32 / kRowsPass, kBatch = kPasses < 4 ? kPasses : 4;
#pragma unroll
    for (int k0 = 0; k0 < kPasses; k0 += kBatch) {
      f32x4_t o[kBatch];
#pragma unroll
      for (int k = 0; k < kBatch; ++k)
        o[k] = *(const f32x4_t*)(mine + ((k0 + k) * kRowsPass + le / kLanesRow) * kYsRow + (le % kLanesRow) * 16);  // 16 bytes: 4 floats or 8 halves
#pragma unroll
      for (int k = 0; k < kBatch; ++k) asm volatile("" : "+v"(o[k]));
#pragma unroll
      for (int k = 0; k < kBatch; ++k) {
        const int r = row_blk + (k0 + k) * kRowsPass + le / kLanesRow;
        if (r < g.it.nrows && cw < g.D && cols_here) {
          f32x4_t* dst = (f32x4_t*)(g.Y + ((size_t)r * g.ldy + b_row0 + (le % kLanesRow) * kColsLane) * kEl);
          if (NT) __builtin_nontemporal_store(o[k], dst);
          else *dst = o[k];
        }
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_sched_barrier(0);
  };
#pragma unroll
  for (int i = NI - 1; i >= 0; --i) out_block(t.acc[i], J, a_row0 + i * 32);
  if constexpr (TALL) out_block(t.accx, t.bx_mode == 3 ? 4 : 2, bx_row0);
}

// What every GEMM-2 workgroup does first (see gemm1_setup).
__device__ __forceinline__ void gemm2_setup(G2Args& g, int item_id, const Layout& L, const char* packed, char* ws, const char* lds, int tid,
                                            int w) {
  g.it = ((const Item2*)(ws + L.o_items2))[item_id];
  const bool sh = g.it.e == L.E_res;
  const int Fp = sh ? L.F_shT : L.Fp;
  const int ld = sh ? L.F_shT : L.F;
  const int KT = ld / kBK;  // stages of the whole expert
  g.KSp = Fp / kBK;         // stages of one partition
  g.np = sh ? 1 : L.P;
  g.D = L.D;
  const char* wbase = sh ? packed + L.p_sw2 + (int64_t)g.it.jd * KT * kStageBytes
                         : packed + L.p_w2 + ((int64_t)g.it.e * L.ND2 + g.it.jd) * KT * kStageBytes;
  const uint16_t* H = sh ? (const uint16_t*)(ws + L.o_Hs) : (const uint16_t*)(ws + L.o_H);
  const int hrow0 = sh ? g.it.row0 : g.it.row0 - L.sh_rows;
  const char* hbase = (const char*)(H + (size_t)hrow0 * ld);
  g.rsW = make_rsrc(wbase, (uint32_t)((int64_t)KT * kStageBytes));
  g.rsH = make_rsrc(hbase, (uint32_t)((int64_t)g.it.nrows * ld * 2));
  const size_t yel = L.yp_half ? 2 : 4;
  if (g.it.split == 0) {  // the item's rows of Yp
    g.Y = ws + L.o_Yp + ((size_t)g.it.row0 * L.D + g.it.jd * kMfmaBN2) * yel;
    g.ldy = L.D;
  } else {  // an extra K range of a split item: a partial-output tile of the pool
    g.Y = ws + L.o_pool + (size_t)(g.it.split - 1) * kPoolRows * kMfmaBN2 * yel;
    g.ldy = kMfmaBN2;
  }
  g.yscale = kYpHalfScale;
  g.h_row_bytes = (uint32_t)(ld * 2);

  g.lds_w = lds_offset(lds) + (uint32_t)(w * 1024);
  g.nstages = 0;
  for (int p = 0; p < g.np; ++p) g.nstages += ((g.it.kmask >> p) & 1) ? g.it.ks_n : 0;
}

// NT: the output leaves with non-temporal stores (for outputs far larger than the caches: the
// combine step reads them from HBM anyway, and the weight and activation tiles keep their place in L2)
template <bool NT, bool YH>
__global__ __launch_bounds__(256) void gemm2_mfma_kernel(Layout L, int T, const char* packed, char* ws) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int item_id = xcd_remap(blockIdx.x);
  if (item_id >= ((const int32_t*)(ws + L.o_counters))[1]) return;  // past the end of the list
  const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid >> 6);
  G2Args g;
  gemm2_setup(g, item_id, L, packed, ws, lds, tid, w);

  if (g.it.nrows > kMfmaBM) {  // a full row tile and the expert's last 1..64 rows
    gemm2_tile<4, 4, 4, NT, YH, RingTall2, true>(g, lds, (w >> 1) * 128, (w & 1) * 128, w);
  } else if (g.it.nrows == kMfmaBM) {
    gemm2_tile<4, 4, 4, NT, YH>(g, lds, (w >> 1) * 128, (w & 1) * 128, w);  // 2 x 2 wavefronts
  } else {  // 1 x 4: the ceil(nrows/32) blocks of pair rows that exist x 64 columns
    switch ((g.it.nrows + 31) >> 5) {
      case 1: gemm2_tile<8, 2, 1, NT, YH>(g, lds, 0, w * 64, w); break;
      case 2: gemm2_tile<8, 2, 2, NT, YH>(g, lds, 0, w * 64, w); break;
      case 3: gemm2_tile<8, 2, 3, NT, YH>(g, lds, 0, w * 64, w); break;
      case 4: gemm2_tile<8, 2, 4, NT, YH>(g, lds, 0, w * 64, w); break;
      case 5: gemm2_tile<8, 2, 5, NT, YH>(g, lds, 0, w * 64, w); break;
      case 6: gemm2_tile<8, 2, 6, NT, YH>(g, lds, 0, w * 64, w); break;
      case 7: gemm2_tile<8, 2, 7, NT, YH>(g, lds, 0, w * 64, w); break;
      default: gemm2_tile<8, 2, 8, NT, YH>(g, lds, 0, w * 64, w); break;
    }
  }
}

static hipError_t set_lds_attr_now() {
  const struct {
    const void* fn;
    int bytes;
  } kernels[] = {
      {(const void*)gemm1_mfma_kernel<false>, kLdsBytes},       {(const void*)gemm1_mfma_kernel<true>, kLdsBytes},
      {(const void*)gemm2_mfma_kernel<false, false>, kLdsBytes}, {(const void*)gemm2_mfma_kernel<true, false>, kLdsBytes},
      {(const void*)gemm2_mfma_kernel<false, true>, kLdsBytes},  {(const void*)gemm2_mfma_kernel<true, true>, kLdsBytes},
  };
  for (const auto& k : kernels) {
    hipError_t e = hipFuncSetAttribute(k.fn, hipFuncAttributeMaxDynamicSharedMemorySize, k.bytes);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}
static hipError_t set_lds_attr() {
  static PerDeviceOnce once;
  return once.run(set_lds_attr_now);
}

// grids are whole chunks of 256 blocks so that the XCD remap is a bijection
hipError_t launch_gemm1_mfma(const Layout& L, int T, const char* packed, const void* x, char* ws, int epi, hipStream_t s) {
  if (T <= 0) return hipSuccess;
  hipError_t e = set_lds_attr();
  if (e != hipSuccess) return e;
  const int g1 = (items1_bound(L, T) + 255) & ~255;
  const uint16_t* xp = (const uint16_t*)x;
  if (epi == 0) gemm1_mfma_kernel<false><<<dim3(g1), dim3(256), kLdsBytes, s>>>(L, T, packed, xp, ws, 0);
  else gemm1_mfma_kernel<true><<<dim3(g1), dim3(256), kLdsBytes, s>>>(L, T, packed, xp, ws, epi);
  return hipGetLastError();
}

hipError_t launch_gemm2_mfma(const Layout& L, int T, const char* packed, char* ws, hipStream_t s) {
  if (T <= 0) return hipSuccess;
  hipError_t e = set_lds_attr();
  if (e != hipSuccess) return e;
  const int g2 = (items2_bound(L, T) + 255) & ~255;
  // per-pair outputs of this batch, at most; beyond the size of the last-level cache they stream
  const int64_t out_bytes = (int64_t)T * (L.K + (L.n_shared > 0 ? 1 : 0)) * L.D * (L.yp_half ? 2 : 4);
  const bool nt = out_bytes > kStreamOutBytes;
  const dim3 grid(g2), block(256);
  if (L.yp_half) {
    if (nt) gemm2_mfma_kernel<true, true><<<grid, block, kLdsBytes, s>>>(L, T, packed, ws);
    else gemm2_mfma_kernel<false, true><<<grid, block, kLdsBytes, s>>>(L, T, packed, ws);
  } else {
    if (nt) gemm2_mfma_kernel<true, false><<<grid, block, kLdsBytes, s>>>(L, T, packed, ws);
    else gemm2_mfma_kernel<false, false><<<grid, block, kLdsBytes, s>>>(L, T, packed, ws);
  }
  return hipGetLastError();
}

}  // namespace dsmoe
