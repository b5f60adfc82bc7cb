// Load-aware threshold selection on the device (Sec. 4.3 of the paper) and the map from a row
// budget to a threshold through the distribution of the normalised scores (Sec. 5.3.3 notes that
// the threshold <-> drop-rate relation is not linear).
//
// Input is the output of a routing pass over the whole router with nothing dropped: expert id and
// normalised score n of every (token, slot) pair.  sel[e][0 .. kSelBins] is the histogram of
// floor(n * kSelBins) over the pairs of expert e (n = 1 falls into the last bin), sel[e][kSelBins+1]
// the pair count of e.  Because kSelBins is a power of two, n * kSelBins is exact in fp32 and
// "n >= b / kSelBins" is the same decision as "bin(n) >= b": suffix sums of the histogram are the
// exact row counts the layer would keep at the grid thresholds.
#include "common.h"

namespace dsmoe {

constexpr int kSelRow = kSelBins + 2;

// row E of sel (when asked for) is the histogram over the pairs of the resident experts [lo, hi)
__global__ __launch_bounds__(256) void score_hist_kernel(const int32_t* __restrict__ idx, const float* __restrict__ n,
                                                         int64_t npairs, int32_t* __restrict__ sel, int E, int lo, int hi,
                                                         int resident_row) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= npairs) return;
  const int e = idx[i];
  int b = (int)floorf(n[i] * (float)kSelBins);
  b = b < 0 ? 0 : (b > kSelBins ? kSelBins : b);
  if (!resident_row) {
    atomicAdd(&sel[(int64_t)e * kSelRow + b], 1);
    atomicAdd(&sel[(int64_t)e * kSelRow + kSelBins + 1], 1);
  } else if (e >= lo && e < hi) {
    atomicAdd(&sel[(int64_t)E * kSelRow + b], 1);
  }
}

// One workgroup per expert.
__global__ __launch_bounds__(256) void tau_pick_kernel(const int32_t* __restrict__ sel, const float* __restrict__ tau_max, int T,
                                                       int E, int K, int P, int G, int row_cap, float* __restrict__ tau,
                                                       int32_t* __restrict__ pair_count) {
  __shared__ int32_t chunk[256];
  __shared__ int32_t s_bin;
  const int e = blockIdx.x, tid = threadIdx.x;
  const int32_t* h = sel + (int64_t)e * kSelRow;
  // load ratio of the device that holds this expert
  const int d0 = (e / G) * G;
  int load = 0;
  for (int j = 0; j < G; ++j) load += sel[(int64_t)(d0 + j) * kSelRow + kSelBins + 1];
  const float ideal = (float)((int64_t)T * K * G) / (float)E;
  const float r = (float)load / ideal;
  const float scale = r < 1.f ? r : 1.f;

  int bstar = 0;
  if (row_cap > 0) {  // smallest b with (pairs of e whose bin >= b) <= row_cap
    constexpr int per = kSelBins / 256;  // bins [tid*per, tid*per+per); the last bin (n = 1) belongs to thread 255
    int sum = 0;
    for (int j = 0; j < per; ++j) sum += h[tid * per + j];
    if (tid == 255) sum += h[kSelBins];
    chunk[tid] = sum;
    if (tid == 0) s_bin = 0;
    __syncthreads();
    int above = 0;  // pairs in the chunks above this thread's
    for (int j = tid + 1; j < 256; ++j) above += chunk[j];
    if (above <= row_cap && above + sum > row_cap) {  // the crossing lies in this chunk: exactly one thread
      int s = above;
      int b = tid == 255 ? kSelBins : tid * per + per - 1;
      for (; b >= tid * per; --b) {
        if (s + h[b] > row_cap) break;
        s += h[b];
      }
      s_bin = b + 1;
    }
    __syncthreads();
    bstar = s_bin;
  }
  if (tid == 0) {
    // one rounding per operation (the multiply must not fuse with the subtraction below)
#pragma clang fp contract(off)
    float lowest = INFINITY;
    for (int p = 0; p < P; ++p) {
      const float v = tau_max[p] * scale;
      lowest = v < lowest ? v : lowest;
    }
    const float floor_e = (float)bstar / (float)kSelBins;
    for (int p = 0; p < P; ++p) {
      float v = tau_max[p] * scale;
      if (floor_e > lowest) v = floor_e + (v - lowest);
      tau[e * P + p] = v;
    }
    if (pair_count) pair_count[e] = h[kSelBins + 1];
  }
}

hipError_t launch_select_thresholds(const Layout& L, int T, const float* tau_max, int group_size, int row_cap, char* ws,
                                    float* tau, int32_t* pair_count, hipStream_t s) {
  int32_t* sel = (int32_t*)(ws + L.o_sel);
  const int64_t npairs = (int64_t)T * L.K;
  if (npairs > 0) {
    score_hist_kernel<<<dim3((unsigned)((npairs + 255) / 256)), dim3(256), 0, s>>>((const int32_t*)(ws + L.o_idx),
                                                                                     (const float*)(ws + L.o_w), npairs, sel, L.E, L.lo, L.hi, 0);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  tau_pick_kernel<<<dim3(L.E), dim3(256), 0, s>>>(sel, tau_max, T, L.E, L.K, L.P, group_size, row_cap, tau, pair_count);
  return hipGetLastError();
}

// Thresholds for a target drop rate (Sec. 5.3.3: the relation between threshold and drop rate is
// read off the batch's own score distribution; Sec. 4.2 c: the partitions keep fixed offsets).
// h = histogram of floor(n * kSelBins) over the resident pairs.  Unit (pair, p) is dropped iff
// n < (b + off[p]) / kSelBins, i.e. iff bin(n) < b + off[p]: with C(x) = pairs whose bin is below x,
// the dropped units at centre b are sum_p C(b + off[p]).  One workgroup: prefix counts in LDS, then
// the smallest b with at least `need` dropped units by bisection (the count grows with b).
struct DropRateArgs {
  int32_t off[kMaxPart];
  int P, E;
  double rate;
};
__global__ __launch_bounds__(1024) void drop_rate_pick_kernel(const int32_t* __restrict__ h, DropRateArgs a,
                                                              float* __restrict__ tau, int32_t* __restrict__ stats) {
  __shared__ int32_t below[kSelBins + 2];  // below[x] = pairs with bin < x, x = 0 .. kSelBins+1
  __shared__ int32_t part[1024];
  const int tid = threadIdx.x;
  constexpr int per = (kSelBins + 1 + 1023) / 1024;  // bins per thread (5)
  int sum = 0;
  for (int j = 0; j < per; ++j) {
    const int b = tid * per + j;
    sum += b <= kSelBins ? h[b] : 0;
  }
  part[tid] = sum;
  __syncthreads();
  for (int o = 1; o < 1024; o <<= 1) {  // inclusive scan of the per-thread sums
    const int v = tid >= o ? part[tid - o] : 0;
    __syncthreads();
    part[tid] += v;
    __syncthreads();
  }
  int run = part[tid] - sum;
  for (int j = 0; j < per; ++j) {
    const int b = tid * per + j;
    if (b <= kSelBins + 1) below[b] = run;
    run += b <= kSelBins ? h[b] : 0;
  }
  __syncthreads();
  if (tid == 0) {
    const int pairs = below[kSelBins + 1];
    auto C = [&](int x) { return x <= 0 ? 0 : (x > kSelBins + 1 ? pairs : below[x]); };
    auto dropped = [&](int b) {
      int d = 0;
      for (int p = 0; p < a.P; ++p) d += C(b + a.off[p]);
      return d;
    };
    int omax = a.off[0], omin = a.off[0];
    for (int p = 1; p < a.P; ++p) {
      omax = max(omax, a.off[p]);
      omin = min(omin, a.off[p]);
    }
    const double need = a.rate * ((double)pairs * a.P);
    int lo_b = -omax, hi_b = kSelBins + 1 - omin;  // nothing dropped .. everything dropped
    while (lo_b < hi_b) {                          // smallest b with dropped(b) >= need
      const int mid = lo_b + ((hi_b - lo_b) >> 1);
      if ((double)dropped(mid) >= need) hi_b = mid;
      else lo_b = mid + 1;
    }
    for (int e = 0; e < a.E; ++e)
      for (int p = 0; p < a.P; ++p) tau[e * a.P + p] = (float)(lo_b + a.off[p]) / (float)kSelBins;
    if (stats) {
      stats[0] = dropped(lo_b);
      stats[1] = pairs * a.P;
    }
  }
}

hipError_t launch_drop_rate_thresholds(const Layout& L, int T, double rate, const int32_t* offset_bins, char* ws, float* tau,
                                       int32_t* stats, hipStream_t s) {
  int32_t* sel = (int32_t*)(ws + L.o_sel);
  const int64_t npairs = (int64_t)T * L.K;
  if (npairs > 0) {
    score_hist_kernel<<<dim3((unsigned)((npairs + 255) / 256)), dim3(256), 0, s>>>((const int32_t*)(ws + L.o_idx),
                                                                                     (const float*)(ws + L.o_w), npairs, sel,
                                                                                     L.E, L.lo, L.hi, 1);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  DropRateArgs a;
  for (int p = 0; p < kMaxPart; ++p) a.off[p] = p < L.P ? offset_bins[p] : 0;
  a.P = L.P;
  a.E = L.E;
  a.rate = rate;
  drop_rate_pick_kernel<<<dim3(1), dim3(1024), 0, s>>>(sel + (int64_t)L.E * kSelRow, a, tau, stats);
  return hipGetLastError();
}

}  // namespace dsmoe
