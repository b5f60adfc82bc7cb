// moe_partition_weights kernels: neuron reorder through perm (Sec. 4.2 b), even split into P
// sub-experts with no W2 scaling (Sec. 3.2), written in the layout the GEMM kernels read.
//
// Generic layout (element type = layer dtype):
//   W1g, W3g [E_res][D][F], W2g [E_res][F][D] with neuron axis in permuted order;
//   shared experts concatenated along the neuron axis: SW1g, SW3g [D][F_shT], SW2g [F_shT][D].
// MFMA layout (bf16): 16 KiB "stage images", each the exact LDS contents of one operand tile of
//   one pipeline stage, rows of kBK = 32 K-values with the 16-byte chunks XOR-rotated (swz_chunk):
//   W13  stage ((e*P + p)*NT1 + jt)*(D/32) + ks : 256 weight rows x 32 values of d; weight row
//        q*64 + gu*32 + j  is neuron  p*Fp + jt*128 + q*32 + j  of W1 (gu=0) or W3 (gu=1): every 64
//        weight rows hold the gate and the up projection of the same 32 neurons
//   W2   stage (e*ND2 + jd)*(F/32) + kt : 256 output columns x 32 neurons (positions kt*32..),
//        as IEEE half precision times 2^s (GEMM-2 multiplies half-precision operands: its left
//        operand, the intermediate activation, needs more significant bits than bf16 has).  s is
//        chosen per layer so that the largest |W2| lands in [2^14, 2^15): every bf16 value within a
//        factor 2^-29 of the largest is then exactly representable (smaller ones round to the
//        subnormal grid, 2^-39 of the largest); the combine kernel multiplies by 2^-s, exactly.
//        The scale record sits at p_scale: uint32 largest |W2| bits, float 2^s, float 2^-(s+k), int32 s.
//   W3 carries the factor 2^k of cfg.h_scale_log2 (exact in bf16), so that the intermediate activation
//        comes out of GEMM-1 times 2^k, in the range half precision resolves best, at no run-time cost.
//   neurons / columns past the end are zero.
#include "common.h"

namespace dsmoe {

template <typename T>
__global__ void pack_generic_kernel(Layout L, const T* w1, const T* w3, const T* w2, const T* sw1, const T* sw3,
                                    const T* sw2, const int32_t* perm, char* packed, int n_shared, int F_sh) {
  const int64_t nW = (int64_t)L.E_res * L.D * L.F;
  const int64_t nS = (int64_t)L.D * L.F_shT;
  const int64_t total = 3 * nW + 3 * nS;
  T* W1g = (T*)(packed + L.p_w13);
  T* W3g = W1g + nW;
  T* W2g = (T*)(packed + L.p_w2);
  T* S1g = (T*)(packed + L.p_sw13);
  T* S3g = S1g + nS;
  T* S2g = (T*)(packed + L.p_sw2);
  for (int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; q < total; q += (int64_t)gridDim.x * blockDim.x) {
    if (q < 2 * nW) {
      const bool up = q >= nW;
      int64_t r = up ? q - nW : q;
      int j = (int)(r % L.F);
      int64_t ed = r / L.F;  // e*D + d
      int e = (int)(ed / L.D);
      int src = perm ? perm[(size_t)e * L.F + j] : j;
      (up ? W3g : W1g)[r] = (up ? w3 : w1)[ed * L.F + src];
    } else if (q < 3 * nW) {
      int64_t r = q - 2 * nW;
      int d = (int)(r % L.D);
      int64_t ej = r / L.D;  // e*F + j
      int e = (int)(ej / L.F), j = (int)(ej % L.F);
      int src = perm ? perm[(size_t)e * L.F + j] : j;
      W2g[r] = w2[((size_t)e * L.F + src) * L.D + d];
    } else if (q < 3 * nW + 2 * nS) {
      int64_t r = q - 3 * nW;
      const bool up = r >= nS;
      if (up) r -= nS;
      int c = (int)(r % L.F_shT);
      int d = (int)(r / L.F_shT);
      int s = c / F_sh, n = c % F_sh;
      (up ? S3g : S1g)[r] = (up ? sw3 : sw1)[((size_t)s * L.D + d) * F_sh + n];
    } else {
      int64_t r = q - 3 * nW - 2 * nS;
      int d = (int)(r % L.D);
      int c = (int)(r / L.D);
      int s = c / F_sh, n = c % F_sh;
      S2g[r] = sw2[((size_t)s * F_sh + n) * L.D + d];
    }
  }
}

// largest finite |w| of a bf16 tensor, as its bit pattern (monotone in the value), into *out
__global__ __launch_bounds__(256) void absmax_bf16_kernel(const uint16_t* w, int64_t n, uint32_t* out) {
  uint32_t m = 0;
  for (int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 8; i < n; i += (int64_t)gridDim.x * 256 * 8) {
    if (i + 8 <= n && (((uintptr_t)(w + i)) & 15) == 0) {
      const uint4 v = *(const uint4*)(w + i);
      const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const uint32_t a = u[k] & 0x7fffu, b = (u[k] >> 16) & 0x7fffu;
        if (a < 0x7f80u && a > m) m = a;
        if (b < 0x7f80u && b > m) m = b;
      }
    } else {
      for (int64_t k = i; k < n && k < i + 8; ++k) {
        const uint32_t a = w[k] & 0x7fffu;
        if (a < 0x7f80u && a > m) m = a;
      }
    }
  }
  for (int o = 32; o > 0; o >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, o, 64));
  if ((threadIdx.x & 63) == 0 && m) atomicMax(out, m);
}

// rec[0] = largest |W2| bits  ->  rec[1] = 2^s, rec[2] = 2^-(s + h_shift), rec[3] = s, with largest * 2^s in
// [2^14, 2^15).  rec[2] undoes both powers of two the packed weights carry: 2^s in W2 and 2^h_shift in W3.
__global__ void w2_scale_kernel(uint32_t* rec, int h_shift) {
  const int e = (int)(rec[0] >> 7);  // biased exponent of the largest value (0: zero or subnormal)
  int s = e == 0 ? 0 : 14 - (e - 127);
  s = s < -80 ? -80 : s > 80 ? 80 : s;
  rec[1] = (uint32_t)(127 + s) << 23;
  rec[2] = (uint32_t)(127 - s - h_shift) << 23;
  rec[3] = (uint32_t)s;
}

// a bf16 value times 2^k (k = L.h_shift), exact unless it leaves bf16's exponent range
__device__ __forceinline__ uint16_t bf16_shift(uint16_t b, int k) {
  return k == 0 ? b : f32_to_bf16(ldexpf(bf16_to_f32(b), k));
}

__device__ __forceinline__ uint16_t bf16_to_scaled_half(uint16_t b, float scale) {
  const _Float16 h = (_Float16)(bf16_to_f32(b) * scale);  // the product is exact; one rounding (none for values in range)
  return __builtin_bit_cast(uint16_t, h);
}

// One thread per 16-byte chunk of the packed MFMA buffers.
__global__ void pack_mfma_kernel(Layout L, const uint16_t* w1, const uint16_t* w3, const uint16_t* w2,
                                 const uint16_t* sw1, const uint16_t* sw3, const uint16_t* sw2, const int32_t* perm,
                                 char* packed, int n_shared, int F_sh, int skip_routed_w13) {
  const int KS1 = L.D / kBK;
  const int64_t chunks_per_stage = kStageBytes / 16;  // 2048
  const int64_t st13 = (int64_t)L.E_res * L.P * L.NT1 * KS1;
  const int64_t st2 = (int64_t)L.E_res * L.ND2 * (L.F / kBK);
  const int64_t sts13 = (int64_t)(n_shared > 0 ? L.NT1_sh * KS1 : 0);
  const int64_t sts2 = (int64_t)(n_shared > 0 ? L.ND2 * (L.F_shT / kBK) : 0);
  const int64_t total = (st13 + st2 + sts13 + sts2) * chunks_per_stage;
  const int64_t first = skip_routed_w13 ? st13 * chunks_per_stage : 0;  // those stages are written by pack_w13_columns_kernel
  for (int64_t q = first + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; q < total; q += (int64_t)gridDim.x * blockDim.x) {
    int64_t stage = q / chunks_per_stage;
    int c = (int)(q % chunks_per_stage);
    const int row = c / kChunksPerRow, pc = c % kChunksPerRow;
    const int lc = swz_chunk(row, pc);  // XOR rotation is its own inverse
    uint16_t v[8];
    char* dst;
    if (stage < st13 + sts13) {
      const bool sh = stage >= st13;
      if (sh) stage -= st13;
      // order of the work: expert, K stage, (partition, neuron tile).  The threads at work at one time
      // then read the same few rows d of W1 / W3 (one 2-byte element per 32-byte sector, in permuted
      // column order), which stay in L2; the destination index below does not depend on this order.
      const int nt1 = sh ? L.NT1_sh : L.NT1;
      const int tiles = (sh ? 1 : L.P) * nt1;
      const int tile = (int)(stage % tiles);
      int64_t r = stage / tiles;
      const int ks = (int)(r % KS1);
      const int e = sh ? 0 : (int)(r / KS1);
      const int jt = tile % nt1;
      const int p = sh ? 0 : tile / nt1;
      const int q = row >> 6, gu = (row >> 5) & 1, j = row & 31;
      const int Fp = sh ? L.F_shT : L.Fp;
      const int nin = jt * kMfmaNeur + q * 32 + j;  // neuron inside the partition
      const int d0 = ks * kBK + lc * 8;
      if (nin < Fp) {
        if (!sh) {
          const int pos = p * Fp + nin;
          const int src = perm ? perm[(size_t)e * L.F + pos] : pos;
          const uint16_t* w = gu ? w3 : w1;
          for (int i = 0; i < 8; ++i) v[i] = bf16_shift(w[((size_t)e * L.D + d0 + i) * L.F + src], gu ? L.h_shift : 0);
        } else {
          const int s = nin / F_sh, n = nin % F_sh;
          const uint16_t* w = gu ? sw3 : sw1;
          for (int i = 0; i < 8; ++i) v[i] = bf16_shift(w[((size_t)s * L.D + d0 + i) * F_sh + n], gu ? L.h_shift : 0);
        }
      } else {
        for (int i = 0; i < 8; ++i) v[i] = 0;
      }
      const int64_t sidx = sh ? ((int64_t)jt * KS1 + ks) : ((((int64_t)e * L.P + p) * L.NT1 + jt) * KS1 + ks);
      dst = packed + (sh ? L.p_sw13 : L.p_w13) + sidx * kStageBytes + (int64_t)c * 16;
    } else {
      stage -= st13 + sts13;
      const bool sh = stage >= st2;
      if (sh) stage -= st2;
      const int KT = (sh ? L.F_shT : L.F) / kBK;
      const int kt = (int)(stage % KT);
      int64_t r = stage / KT;
      const int jd = (int)(r % L.ND2);
      const int e = sh ? 0 : (int)(r / L.ND2);
      const int d = jd * kMfmaBN2 + row;
      const int pos0 = kt * kBK + lc * 8;
      const float w2_scale = ((const float*)(packed + L.p_scale))[1];
      if (d < L.D) {
        for (int i = 0; i < 8; ++i) {
          const int pos = pos0 + i;
          if (!sh) {
            const int src = perm ? perm[(size_t)e * L.F + pos] : pos;
            v[i] = bf16_to_scaled_half(w2[((size_t)e * L.F + src) * L.D + d], w2_scale);
          } else {
            const int s = pos / F_sh, n = pos % F_sh;
            v[i] = bf16_to_scaled_half(sw2[((size_t)s * F_sh + n) * L.D + d], w2_scale);
          }
        }
      } else {
        for (int i = 0; i < 8; ++i) v[i] = 0;
      }
      const int64_t sidx = sh ? ((int64_t)jd * KT + kt) : (((int64_t)e * L.ND2 + jd) * KT + kt);
      dst = packed + (sh ? L.p_sw2 : L.p_w2) + sidx * kStageBytes + (int64_t)c * 16;
    }
    uint4 o;
    o.x = v[0] | ((uint32_t)v[1] << 16);
    o.y = v[2] | ((uint32_t)v[3] << 16);
    o.z = v[4] | ((uint32_t)v[5] << 16);
    o.w = v[6] | ((uint32_t)v[7] << 16);
    *(uint4*)dst = o;
  }
}

// The routed W1 / W3 stages, walked in SOURCE order: a thread takes one original neuron (column
// src of W1 and W3) and one K stage, reads its 32 values of d from 32 rows (neighbouring threads read
// neighbouring columns: whole cache lines, where a walk in destination order fetches a line per
// 2-byte element of a permuted column) and writes the neuron's two 64-byte image rows at the place
// the inverse permutation names.  inv == nullptr: identity order.
__global__ __launch_bounds__(256) void pack_w13_columns_kernel(Layout L, const uint16_t* w1, const uint16_t* w3, const int32_t* inv,
                                                              char* packed) {
  const int src = blockIdx.x * 256 + threadIdx.x, ks = blockIdx.y, e = blockIdx.z;
  if (src >= L.F) return;
  const int pos = inv ? inv[(size_t)e * L.F + src] : src;
  const int p = pos / L.Fp, nin = pos % L.Fp;
  const int jt = nin / kMfmaNeur, q = (nin % kMfmaNeur) >> 5, j = nin & 31;
  const int KS1 = L.D / kBK;
  char* stage = packed + L.p_w13 + ((((int64_t)e * L.P + p) * L.NT1 + jt) * KS1 + ks) * kStageBytes;
#pragma unroll
  for (int gu = 0; gu < 2; ++gu) {
    const uint16_t* w = (gu ? w3 : w1) + ((size_t)e * L.D + (size_t)ks * kBK) * L.F + src;
    uint16_t v[kBK];
#pragma unroll
    for (int i = 0; i < kBK; ++i) v[i] = bf16_shift(w[(size_t)i * L.F], gu ? L.h_shift : 0);
    const int row = q * 64 + gu * 32 + j;
#pragma unroll
    for (int lc = 0; lc < kChunksPerRow; ++lc) {
      uint4 o;
      o.x = v[8 * lc + 0] | ((uint32_t)v[8 * lc + 1] << 16);
      o.y = v[8 * lc + 2] | ((uint32_t)v[8 * lc + 3] << 16);
      o.z = v[8 * lc + 4] | ((uint32_t)v[8 * lc + 5] << 16);
      o.w = v[8 * lc + 6] | ((uint32_t)v[8 * lc + 7] << 16);
      *(uint4*)(stage + row * (kBK * 2) + swz_chunk(row, lc) * 16) = o;
    }
  }
}

// image rows of the neurons past the end of a partition (its last neuron tile is not full): zeros
__global__ __launch_bounds__(256) void pack_w13_padding_kernel(Layout L, char* packed) {
  const int pad = L.NT1 * kMfmaNeur - L.Fp;  // neurons per (expert, partition) that do not exist
  const int KS1 = L.D / kBK;
  const int64_t total = (int64_t)L.E_res * L.P * KS1 * pad * 2 * kChunksPerRow;
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= total) return;
  const int pc = (int)(t % kChunksPerRow);
  int64_t r = t / kChunksPerRow;
  const int gu = (int)(r % 2);
  r /= 2;
  const int nin = L.Fp + (int)(r % pad);
  r /= pad;
  const int ks = (int)(r % KS1);
  const int64_t ep = r / KS1;  // e * P + p
  const int jt = nin / kMfmaNeur, q = (nin % kMfmaNeur) >> 5, j = nin & 31;
  const int row = q * 64 + gu * 32 + j;
  char* stage = packed + L.p_w13 + ((ep * L.NT1 + jt) * KS1 + ks) * kStageBytes;
  *(uint4*)(stage + row * (kBK * 2) + pc * 16) = make_uint4(0, 0, 0, 0);
}

// inv[e][perm[e][pos]] = pos
__global__ void invert_perm_kernel(const int32_t* perm, int32_t* inv, int F, int64_t n) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n) return;
  const int64_t e = t / F;
  const int src = perm[t];
  if (src >= 0 && src < F) inv[e * F + src] = (int32_t)(t % F);  // a bad perm is refused before this runs; stay in bounds regardless
}

hipError_t launch_pack(const Layout& L, const void* w1, const void* w3, const void* w2, const void* sw1, const void* sw3,
                       const void* sw2, const int32_t* perm, char* packed, int n_shared, int F_sh, hipStream_t s) {
  dim3 block(256), grid(256 * 64);
  if (L.mfma) {
    // the layer's W2 scale (see the layout comment at the top), from the largest |W2| of routed and shared experts
    uint32_t* rec = (uint32_t*)(packed + L.p_scale);
    hipError_t e0 = launch_fill_i32((int32_t*)rec, 4, 0, s);
    if (e0 != hipSuccess) return e0;
    absmax_bf16_kernel<<<dim3(2048), dim3(256), 0, s>>>((const uint16_t*)w2, (int64_t)L.E_res * L.F * L.D, rec);
    if (n_shared > 0) absmax_bf16_kernel<<<dim3(512), dim3(256), 0, s>>>((const uint16_t*)sw2, (int64_t)L.F_shT * L.D, rec);
    w2_scale_kernel<<<dim3(1), dim3(1), 0, s>>>(rec, L.h_shift);
    // The routed W1 / W3 stages are written in source order (see pack_w13_columns_kernel), which
    // needs the inverse permutation: it is parked in the W2 region of the packed buffer, which
    // the last kernel overwrites.  (That region has E_res * F * D * 2 bytes, the table E_res * F * 4.)
    const bool columns = L.D >= 2 && (int64_t)L.D / kBK <= 65535 && L.E_res <= 65535;
    if (columns) {
      int32_t* inv = nullptr;
      if (perm) {
        inv = (int32_t*)(packed + L.p_w2);
        const int64_t n = (int64_t)L.E_res * L.F;
        invert_perm_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s>>>(perm, inv, L.F, n);
      }
      pack_w13_columns_kernel<<<dim3((L.F + 255) / 256, L.D / kBK, L.E_res), dim3(256), 0, s>>>(
          L, (const uint16_t*)w1, (const uint16_t*)w3, inv, packed);
      const int pad = L.NT1 * kMfmaNeur - L.Fp;
      if (pad > 0) {
        const int64_t total = (int64_t)L.E_res * L.P * (L.D / kBK) * pad * 2 * kChunksPerRow;
        pack_w13_padding_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s>>>(L, packed);
      }
    }
    pack_mfma_kernel<<<grid, block, 0, s>>>(L, (const uint16_t*)w1, (const uint16_t*)w3, (const uint16_t*)w2,
                                            (const uint16_t*)sw1, (const uint16_t*)sw3, (const uint16_t*)sw2, perm, packed,
                                            n_shared, F_sh > 0 ? F_sh : 1, columns ? 1 : 0);
  } else if (L.dtype == DSMOE_F32) {
    pack_generic_kernel<float><<<grid, block, 0, s>>>(L, (const float*)w1, (const float*)w3, (const float*)w2,
                                                      (const float*)sw1, (const float*)sw3, (const float*)sw2, perm, packed,
                                                      n_shared, F_sh > 0 ? F_sh : 1);
  } else {
    pack_generic_kernel<uint16_t><<<grid, block, 0, s>>>(L, (const uint16_t*)w1, (const uint16_t*)w3, (const uint16_t*)w2,
                                                         (const uint16_t*)sw1, (const uint16_t*)sw3, (const uint16_t*)sw2,
                                                         perm, packed, n_shared, F_sh > 0 ? F_sh : 1);
  }
  return hipGetLastError();
}

// perm check: scratch[0 .. E_res*F) counts how often each neuron id is named (zeroed by the
// caller), scratch[E_res*F] counts violations (out of range or named twice).
__global__ void perm_check_kernel(Layout L, const int32_t* perm, int32_t* scratch) {
  const int64_t n = (int64_t)L.E_res * L.F;
  const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (q >= n) return;
  const int e = (int)(q / L.F);
  const int v = perm[q];
  if (v < 0 || v >= L.F) {
    atomicAdd(&scratch[n], 1);
  } else if (atomicAdd(&scratch[(size_t)e * L.F + v], 1) != 0) {
    atomicAdd(&scratch[n], 1);
  }
}

hipError_t launch_perm_check(const Layout& L, const int32_t* perm, int32_t* scratch, hipStream_t s) {
  const int64_t n = (int64_t)L.E_res * L.F;
  hipError_t err = launch_fill_i32(scratch, n + 1, 0, s);
  if (err != hipSuccess) return err;
  perm_check_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s>>>(L, perm, scratch);
  return hipGetLastError();
}

}  // namespace dsmoe
