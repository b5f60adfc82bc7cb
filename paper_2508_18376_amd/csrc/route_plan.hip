// Gating + drop mask, row-list construction (histogram, scan, scatter) and the combine kernel.
//
// Gating follows Eq. 1-2 of the paper (softmax over all E logits, Top-K), the mask follows
// Sec. 4.1 / 4.2 c (normalise the K selected scores, keep unit (t,k,p) iff n >= tau[e][p]).
// The row lists realise the index remap of Sec. 3.2 without materialising K*P lists: the pairs of
// one expert are sorted by their keep pattern, so the rows that need sub-expert p are (for
// thresholds that grow with p) a prefix of the expert's list.
#include "common.h"

namespace dsmoe {

// ------------------------------------------------------------------------------------- fill
__global__ void fill_i32_kernel(int32_t* p, int64_t n, int32_t v) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}
hipError_t launch_fill_i32(int32_t* p, int64_t n, int32_t v, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  fill_i32_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s>>>(p, n, v);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------- route
struct RouteArgs {
  const float* logits;
  const float* tau;
  int32_t* idx;
  float* w;
  uint8_t* keep;
  int32_t* bin_count;    // forward: [blocks][nbins] sort-bin histogram, one row per block (may be null)
  int32_t* group_count;  // stand-alone: [E*P] kept units per sub-expert (may be null)
  int T, E, K, P, lo, hi, renorm, nsub_bits, nsub, nhist;
};

// sort bin of a keep pattern inside its expert: patterns that keep the major partitions come first
__device__ __forceinline__ int sub_of_bits(int bits, int nsub_bits) {
  int rev = 0;
  for (int p = 0; p < nsub_bits; ++p) rev |= ((bits >> p) & 1) << (nsub_bits - 1 - p);
  return (1 << nsub_bits) - 1 - rev;
}

// tau: the [E][P] threshold table (the sixteen-lanes-per-token kernel keeps a copy in LDS)
__device__ __forceinline__ int keep_bits_of(float n, int e, const RouteArgs& a, const float* tau) {
  int bits = 0;
  if (e >= a.lo && e < a.hi) {
    for (int p = 0; p < a.P; ++p) bits |= (n >= tau[e * a.P + p] ? 1 : 0) << p;
  }
  return bits;
}

// histogram update of one pair into the block's LDS histogram
__device__ __forceinline__ void count_pair(int32_t* hist, int bits, int e, const RouteArgs& a) {
  if (bits == 0) return;
  if (a.bin_count) atomicAdd(&hist[(e - a.lo) * a.nsub + sub_of_bits(bits, a.nsub_bits)], 1);
  if (a.group_count) {
    int32_t* h2 = hist + (a.bin_count ? (a.hi - a.lo) * a.nsub : 0);
    for (int p = 0; p < a.P; ++p)
      if ((bits >> p) & 1) atomicAdd(&h2[e * a.P + p], 1);
  }
}

// One lane per token; all E logits of the token live in that lane's registers (E <= EPAD <= 32).
template <int EPAD, int KMAX>
__global__ __launch_bounds__(64) void route_lane_kernel(RouteArgs a) {
  extern __shared__ int32_t hist[];
  for (int i = threadIdx.x; i < a.nhist; i += 64) hist[i] = 0;
  __syncthreads();
  const int t = blockIdx.x * 64 + threadIdx.x;
  if (t < a.T) {
    float l[EPAD];
#pragma unroll
    for (int e = 0; e < EPAD; ++e) l[e] = (e < a.E) ? a.logits[(size_t)t * a.E + e] : -INFINITY;
    float m = l[0];
#pragma unroll
    for (int e = 1; e < EPAD; ++e) m = (e < a.E && l[e] > m) ? l[e] : m;
    float z = 0.f;
#pragma unroll
    for (int e = 0; e < EPAD; ++e)
      if (e < a.E) z += expf(l[e] - m);
    // Top-K: K rounds of "largest not yet taken"; a later index wins only if strictly larger.
    float sk[KMAX];
    int ik[KMAX];
    unsigned long long taken = 0ull;
    float sel = 0.f;
#pragma unroll
    for (int k = 0; k < KMAX; ++k) {
      sk[k] = 0.f;
      ik[k] = 0;
      if (k < a.K) {
        float bv = 0.f;
        int be = -1;
#pragma unroll
        for (int e = 0; e < EPAD; ++e) {
          bool free_e = (e < a.E) && !((taken >> e) & 1ull);
          if (free_e && (be < 0 || l[e] > bv)) {
            bv = l[e];
            be = e;
          }
        }
        taken |= 1ull << be;
        ik[k] = be;
        sk[k] = expf(bv - m) / z;  // Eq. 1
        sel += sk[k];
      }
    }
#pragma unroll
    for (int k = 0; k < KMAX; ++k) {
      if (k < a.K) {
        float n = sk[k] / sel;  // Sec. 4.1: normalise over the K selected
        int bits = keep_bits_of(n, ik[k], a, a.tau);
        size_t o = (size_t)t * a.K + k;
        a.idx[o] = ik[k];
        a.w[o] = a.renorm ? n : sk[k];
        a.keep[o] = (uint8_t)bits;
        count_pair(hist, bits, ik[k], a);
      }
    }
  }
  __syncthreads();
  const int nb = a.bin_count ? (a.hi - a.lo) * a.nsub : 0;
  for (int i = threadIdx.x; i < a.nhist; i += 64) {
    int c = hist[i];
    if (i < nb) a.bin_count[(size_t)blockIdx.x * nb + i] = c;  // this block's row of the histogram: no atomics
    else if (c) atomicAdd(&a.group_count[i - nb], c);
  }
}

// Sixteen lanes per token (one row of the wavefront), NCH * 4 logits per lane: lane r of the row
// holds experts 64c + 4r .. 64c + 4r + 3 of every chunk c of 64 experts (16-byte loads, 256
// contiguous bytes per row and chunk).  All reductions stay inside a row: four data-parallel
// steps (mirror, half mirror, two quad permutations) leave the result in every lane, with no
// scalar round trip, and the four rows of a wavefront work on four tokens at once.  U tokens per
// row are carried through every step together so that their dependency chains overlap.
// A block is WV wavefronts = WV * 4 * U tokens.
__device__ __forceinline__ int row_min(int v) {
  v = min(v, dpp_all<kRowMirror>(v));
  v = min(v, dpp_all<kRowHalfMirror>(v));
  v = min(v, dpp_all<kQuadSwap2>(v));
  v = min(v, dpp_all<kQuadSwap1>(v));
  return v;
}

template <int NCH, int U, int WV>
__global__ __launch_bounds__(WV * 64) void route_row_kernel(RouteArgs a) {
  constexpr int kThreads = WV * 64, kTokens = WV * 4 * U, V = NCH * 4;
  extern __shared__ int32_t hist[];
  for (int i = threadIdx.x; i < a.nhist; i += kThreads) hist[i] = 0;
  // the threshold table is fetched now, together with the logits, not after the scores are known
  float* tau_l = (float*)(hist + a.nhist);
  for (int i = threadIdx.x; i < a.E * a.P; i += kThreads) tau_l[i] = a.tau[i];
  // (the barrier that publishes hist and tau_l sits right before their first use, after the scores)
  const int r = threadIdx.x & 15, row = threadIdx.x >> 4;  // lane in its row; row in the block (WV * 4 of them)
  const int t_end = min(a.T, ((int)blockIdx.x + 1) * kTokens);
  auto token = [&](int u) { return (int)blockIdx.x * kTokens + u * (WV * 4) + row; };
  auto expert = [&](int j) { return 64 * (j >> 2) + 4 * r + (j & 3); };
  float l[U][V];
  const bool vec = (a.E & 3) == 0;  // rows of the logits are 16-byte aligned
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int t = token(u);
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int e0 = 64 * c + 4 * r;
      float4 v = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
      if (t < t_end) {
        const float* src = a.logits + (size_t)t * a.E + e0;
        if (vec) {
          if (e0 < a.E) v = *(const float4*)src;
        } else {
          if (e0 + 0 < a.E) v.x = src[0];
          if (e0 + 1 < a.E) v.y = src[1];
          if (e0 + 2 < a.E) v.z = src[2];
          if (e0 + 3 < a.E) v.w = src[3];
        }
      }
      // a NaN logit ranks last, so every round below finds a winner
      l[u][4 * c + 0] = v.x != v.x ? -INFINITY : v.x;
      l[u][4 * c + 1] = v.y != v.y ? -INFINITY : v.y;
      l[u][4 * c + 2] = v.z != v.z ? -INFINITY : v.z;
      l[u][4 * c + 3] = v.w != v.w ? -INFINITY : v.w;
    }
  }
  float m[U], z[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    float v = l[u][0];
#pragma unroll
    for (int j = 1; j < V; ++j) v = fmaxf(v, l[u][j]);
    m[u] = row_max(v);
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    float v = 0.f;
#pragma unroll
    for (int j = 0; j < V; ++j)
      if (expert(j) < a.E) v += expf(l[u][j] - m[u]);
    z[u] = row_sum(v);
  }
  // Top-K in K rounds of "largest logit not yet taken, lowest expert id among equals" (Eq. 2): the
  // row's maximum, then the row's smallest expert id among the lanes that hold it; slot k of the
  // token is round k's winner.  rank = slot of a selected logit, a.K for the others.
  int rank[U][V];
  uint32_t taken[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    taken[u] = 0;
#pragma unroll
    for (int j = 0; j < V; ++j) {
      rank[u][j] = a.K;
      if (expert(j) >= a.E) taken[u] |= 1u << j;
    }
  }
  for (int k = 0; k < a.K; ++k) {
    float g[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float v = -INFINITY;
#pragma unroll
      for (int j = 0; j < V; ++j) v = fmaxf(v, (taken[u] >> j) & 1 ? -INFINITY : l[u][j]);
      g[u] = row_max(v);
    }
    int win[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      int cand = 0x7fffffff;
#pragma unroll
      for (int j = V - 1; j >= 0; --j)  // expert ids grow with j: the last assignment is the smallest
        if (!((taken[u] >> j) & 1) && l[u][j] == g[u]) cand = expert(j);
      win[u] = row_min(cand);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int j = 0; j < V; ++j)
        if (expert(j) == win[u]) {
          rank[u][j] = k;
          taken[u] |= 1u << j;
        }
    }
  }
  float sc[U][V], ssum[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    float v = 0.f;
#pragma unroll
    for (int j = 0; j < V; ++j) {
      const bool selq = expert(j) < a.E && rank[u][j] < a.K;
      sc[u][j] = selq ? expf(l[u][j] - m[u]) / z[u] : 0.f;  // Eq. 1
      v += sc[u][j];
    }
    ssum[u] = row_sum(v);
  }
  __syncthreads();  // hist is cleared and tau_l is complete
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int t = token(u);
    if (t >= t_end) continue;
#pragma unroll
    for (int j = 0; j < V; ++j) {
      const int e = expert(j);
      if (e < a.E && rank[u][j] < a.K) {
        const float n = sc[u][j] / ssum[u];  // Sec. 4.1: normalise over the K selected
        const int bits = keep_bits_of(n, e, a, tau_l);
        const size_t o = (size_t)t * a.K + rank[u][j];
        a.idx[o] = e;
        a.w[o] = a.renorm ? n : sc[u][j];
        a.keep[o] = (uint8_t)bits;
        count_pair(hist, bits, e, a);
      }
    }
  }
  __syncthreads();
  const int nb = a.bin_count ? (a.hi - a.lo) * a.nsub : 0;
  for (int i = threadIdx.x; i < a.nhist; i += kThreads) {
    int c = hist[i];
    if (i < nb) a.bin_count[(size_t)blockIdx.x * nb + i] = c;  // this block's row of the histogram: no atomics
    else if (c) atomicAdd(&a.group_count[i - nb], c);
  }
}

hipError_t launch_route(const Layout& L, const float* logits, int T, const float* tau, int32_t* idx, float* w,
                        uint8_t* keep, int32_t* bin_count, int32_t* group_count, hipStream_t s, bool whole_router_scores) {
  if (T <= 0) return hipSuccess;
  RouteArgs a;
  a.logits = logits;
  a.tau = tau;
  a.idx = idx;
  a.w = w;
  a.keep = keep;
  a.bin_count = bin_count;
  a.group_count = group_count;
  a.T = T;
  a.E = L.E;
  a.K = L.K;
  a.P = L.P;
  // whole_router_scores: every expert counts as resident and w receives the normalised score
  a.lo = whole_router_scores ? 0 : L.lo;
  a.hi = whole_router_scores ? L.E : L.hi;
  a.renorm = whole_router_scores ? 1 : L.renorm;
  a.nsub = L.nsub;
  a.nsub_bits = L.P < kSubBits ? L.P : kSubBits;
  a.nhist = (bin_count ? L.nbins : 0) + (group_count ? L.E * L.P : 0);
  const size_t sh = sizeof(int32_t) * (size_t)(a.nhist + L.E * L.P);  // histogram + (row kernel) threshold table
  if (L.E <= 32) {  // few experts: a lane per token, no cross-lane traffic
    dim3 grid((T + 63) / 64), block(64);
    if (L.E <= 8) route_lane_kernel<8, 8><<<grid, block, sh, s>>>(a);
    else if (L.E <= 16) route_lane_kernel<16, 16><<<grid, block, sh, s>>>(a);
    else route_lane_kernel<32, 16><<<grid, block, sh, s>>>(a);
  } else if (T > kWaveSmallBatch) {  // many experts: sixteen lanes per token, 64 tokens per block
    dim3 grid((T + kRouteBlockTokens - 1) / kRouteBlockTokens);
    if (L.E <= 64) route_row_kernel<1, 1, 16><<<grid, dim3(1024), sh, s>>>(a);
    else if (L.E <= 128) route_row_kernel<2, 1, 16><<<grid, dim3(1024), sh, s>>>(a);
    else if (L.E <= 256) route_row_kernel<4, 1, 16><<<grid, dim3(1024), sh, s>>>(a);
    else route_row_kernel<8, 1, 16><<<grid, dim3(1024), sh, s>>>(a);
  } else {  // small batch: 16 tokens per block, one per row of four wavefronts
    dim3 grid((T + kWaveBlockTokens - 1) / kWaveBlockTokens), block(256);
    if (L.E <= 64) route_row_kernel<1, 1, 4><<<grid, block, sh, s>>>(a);
    else if (L.E <= 128) route_row_kernel<2, 1, 4><<<grid, block, sh, s>>>(a);
    else if (L.E <= 256) route_row_kernel<4, 1, 4><<<grid, block, sh, s>>>(a);
    else route_row_kernel<8, 1, 4><<<grid, block, sh, s>>>(a);
  }
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------- plan
// Single-workgroup kernel: turns the bin histogram into row offsets, the row-tile table and the
// two work lists of the grouped GEMMs.  Everything stays on the device: the GEMM grids are sized
// for the worst case and read their item count from the counters this kernel writes.
constexpr int kPlanThreads = 1024;
constexpr int kPlanTilesLds = 2048;  // row tiles whose keep patterns fit in the plan kernel's LDS

// exclusive scan of a[0..n) in LDS (n <= 8 * kPlanThreads); returns the total. tmp: kPlanThreads ints.
// Each thread owns a run of elements; the runs are scanned inside each wavefront with lane shifts
// and the sixteen wavefront totals by the first wavefront: three barriers in all (one for short arrays).
__device__ int block_excl_scan(int32_t* a, int n, int32_t* tmp) {
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  if (n <= 512) {  // short arrays (experts, groups): the first wavefront alone, one barrier
    if (wv == 0) {
      const int per = (n + 63) >> 6;
      const int lo = lane * per, hi = min(n, lo + per);
      int sum = 0;
      for (int i = lo; i < hi; ++i) sum += a[i];
      int incl = sum;
      for (int o = 1; o < 64; o <<= 1) {
        const int v = __shfl_up(incl, o, 64);
        if (lane >= o) incl += v;
      }
      int run = incl - sum;
      for (int i = lo; i < hi; ++i) {
        const int v = a[i];
        a[i] = run;
        run += v;
      }
      if (lane == 63) tmp[128] = incl;
    }
    __syncthreads();
    return tmp[128];
  }
  const int per = (n + kPlanThreads - 1) / kPlanThreads;
  const int lo = tid * per, hi = min(n, lo + per);
  int sum = 0;
  for (int i = lo; i < hi; ++i) sum += a[i];
  int incl = sum;  // inclusive scan over the lanes of this wavefront
  for (int o = 1; o < 64; o <<= 1) {
    const int v = __shfl_up(incl, o, 64);
    if (lane >= o) incl += v;
  }
  if (lane == 63) tmp[wv] = incl;
  __syncthreads();
  if (wv == 0) {
    const int t = lane < kPlanThreads / 64 ? tmp[lane] : 0;
    int inc = t;
    for (int o = 1; o < kPlanThreads / 64; o <<= 1) {
      const int v = __shfl_up(inc, o, 64);
      if (lane >= o) inc += v;
    }
    if (lane < kPlanThreads / 64) tmp[64 + lane] = inc - t;  // exclusive offset of each wavefront
    if (lane == kPlanThreads / 64 - 1) tmp[128] = inc;       // grand total
  }
  __syncthreads();
  int run = tmp[64 + wv] + incl - sum;
  const int total = tmp[128];
  for (int i = lo; i < hi; ++i) {
    const int v = a[i];
    a[i] = run;
    run += v;
  }
  __syncthreads();
  return total;
}

__global__ __launch_bounds__(kPlanThreads) void plan_kernel(Layout L, int T, char* ws) {
  extern __shared__ int32_t sm[];
  // 0. column sums of the route kernel's per-block histograms -> bins[] in LDS
  int32_t* bin_count = sm;  // [nbins]
  {
    const int32_t* blk_hist = (const int32_t*)(ws + L.o_bin_count);
    const int nblk = (T + route_block_tokens(L.E, T) - 1) / route_block_tokens(L.E, T);
    // rows r0, r0 + step, .. of column c, eight independent loads at a time (the sum is latency bound)
    auto col_sum = [&](int c, int r0, int step) {
      const int32_t* col = blk_hist + c;
      int sum = 0, r = r0;
      for (; r + 7 * step < nblk; r += 8 * step) {
        int v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = col[(size_t)(r + u * step) * L.nbins];
#pragma unroll
        for (int u = 0; u < 8; ++u) sum += v[u];
      }
      for (; r < nblk; r += step) sum += col[(size_t)r * L.nbins];
      return sum;
    };
    const int G = kPlanThreads / L.nbins;  // threads that share a column (0: more columns than threads)
    if (G <= 1) {
      for (int c = threadIdx.x; c < L.nbins; c += kPlanThreads) bin_count[c] = col_sum(c, 0, 1);
    } else {
      for (int i = threadIdx.x; i < L.nbins; i += kPlanThreads) bin_count[i] = 0;
      __syncthreads();
      const int c = threadIdx.x % L.nbins, g = threadIdx.x / L.nbins;
      if (g < G) {
        const int sum = col_sum(c, g, G);
        if (sum) atomicAdd(&bin_count[c], sum);
      }
    }
    __syncthreads();
  }
  const int tid = threadIdx.x;
  // Two workgroups: both work out the tables that the lists are made from (row counts, tile patterns, short
  // last tiles); then workgroup 0 writes the GEMM-2 list and workgroup 1 the GEMM-1 list, side by side.
  const bool lists2 = blockIdx.x == 0, lists1 = !lists2;
  const int E_res = L.E_res;
  const int has_sh = L.n_shared > 0 ? 1 : 0;
  const int E_tot = E_res + has_sh;
  const int NG = E_tot * L.P;  // (expert, partition) groups; the shared pseudo-expert only uses p = 0
  int32_t* ne = sm + L.nbins;       // [E_tot] rows of each expert
  int32_t* rs = ne + E_tot + 1;     // [E_tot] first row (tile aligned)
  int32_t* ts = rs + E_tot + 1;     // [E_tot] first tile
  int32_t* pt = ts + E_tot + 1;     // [E_tot+1] first tile by POSITION in the row space
  int32_t* ga = pt + E_tot + 2;     // [NG] active tiles of each group
  int32_t* gb = ga + NG + 1;        // [NG+1] item base of each group
  int32_t* abp = gb + NG + 1;       // [E_tot+1] by POSITION: short last tiles (absorbed by tall items) of the experts before
  int32_t* tmp = abp + E_tot + 2;   // [kPlanThreads]

  int32_t* cursor = (int32_t*)(ws + L.o_cursor);
  int32_t* exp_nrows = (int32_t*)(ws + L.o_exp_nrows);
  int32_t* exp_row0 = (int32_t*)(ws + L.o_exp_row0);
  int32_t* counters = (int32_t*)(ws + L.o_counters);
  int32_t* act_rank = (int32_t*)(ws + L.o_act_rank);
  Item1* items1 = (Item1*)(ws + L.o_items1);
  Item2* items2 = (Item2*)(ws + L.o_items2);
  const int BM = L.BM;
  const int bm_sh = 31 - __clz(BM);  // the tile heights are powers of two
  auto tiles_of = [&](int rows) { return (rows + BM - 1) >> bm_sh; };
  const int nsub_bits = L.P < kSubBits ? L.P : kSubBits;

  // 1. rows per expert.  Order of the experts in the row space: the shared pseudo-expert first
  //    (its size is known without the histogram), then the resident experts by id.
  //    position i -> expert: with shared experts, position 0 is id E_res and position i is id i-1.
  for (int e = tid; e < E_tot; e += kPlanThreads) {
    int n = 0;
    if (e < E_res)
      for (int sb = 0; sb < L.nsub; ++sb) n += bin_count[e * L.nsub + sb];
    else
      n = T;
    ne[e] = n;
  }
  __syncthreads();
  // 2. tile-aligned row starts: exclusive scan of the tile counts in position order
  for (int i = tid; i < E_tot; i += kPlanThreads) {
    int e = has_sh ? (i == 0 ? E_res : i - 1) : i;
    pt[i] = tiles_of(ne[e]);
  }
  __syncthreads();
  const int total_tiles = block_excl_scan(pt, E_tot, tmp);
  if (tid == 0) pt[E_tot] = total_tiles;
  for (int i = tid; i < E_tot; i += kPlanThreads) {
    int e = has_sh ? (i == 0 ? E_res : i - 1) : i;
    ts[e] = pt[i];
    rs[e] = pt[i] * BM;
  }
  __syncthreads();
  if (lists2) {
    for (int e = tid; e < E_res; e += kPlanThreads) {
      exp_nrows[e] = ne[e];
      exp_row0[e] = rs[e];
    }
  }
  // 3. first row of every bin; the scatter kernel's cursors start there
  if (lists2) {
    for (int b = tid; b < L.nbins; b += kPlanThreads) {
      int e = b / L.nsub, sb = b % L.nsub;
      int off = rs[e];
      for (int s2 = 0; s2 < sb; ++s2) off += bin_count[e * L.nsub + s2];
      cursor[b] = off;
    }
  }
  // 4. row tiles are described on the fly from the LDS tables (no round trip through global memory):
  //    tile g belongs to the expert at the last position whose first tile is <= g
  auto tile_expert = [&](int g) {
    int lo_i = 0, hi_i = E_tot;  // first position with pt > g
    while (lo_i < hi_i) {
      int mid = (lo_i + hi_i) >> 1;
      if (pt[mid] > g) hi_i = mid;
      else lo_i = mid + 1;
    }
    const int pos = lo_i - 1;
    return has_sh ? (pos == 0 ? E_res : pos - 1) : pos;
  };
  // partitions kept by some row of tile i of expert e (OR of the keep patterns of the bins it overlaps)
  auto tile_bits_of = [&](int e, int i) {
    if (e >= E_res) return 1;
    const int r0 = i * BM, r1 = min(ne[e], r0 + BM);
    int bits = 0, off = 0;
    for (int sb = 0; sb < L.nsub; ++sb) {
      int c = bin_count[e * L.nsub + sb];
      if (c > 0 && off < r1 && off + c > r0) {
        int rev = L.nsub - 1 - sb;
        int pat = 0;
        for (int p = 0; p < nsub_bits; ++p) pat |= ((rev >> (nsub_bits - 1 - p)) & 1) << p;
        if (L.P > nsub_bits) pat |= ((1 << L.P) - 1) & ~((1 << nsub_bits) - 1);  // partitions outside the sort key: assume kept
        bits |= pat;
      }
      off += c;
    }
    return bits;
  };
  // the keep pattern of every row tile, worked out once and in parallel (the per-group loop of
  // step 6 walks the tiles of an expert one after the other and must not redo this for each)
  // (kept in LDS when there are at most kPlanTilesLds tiles, else in the workspace)
  int32_t* tbits = total_tiles <= kPlanTilesLds ? tmp + kPlanThreads : (int32_t*)(ws + L.o_tile_bits);
  for (int g = tid; g < total_tiles; g += kPlanThreads) {
    const int e = tile_expert(g);
    tbits[g] = tile_bits_of(e, g - ts[e]);
  }
  __shared__ int est[4];  // see "tall GEMM-1 items" below
  if (tid < 4) est[tid] = 0;
  __syncthreads();
  // rows of tile i of expert e up to the last one that keeps partition p.  The rows are sorted by
  // keep pattern, so with thresholds that grow with p this is exactly the number of rows that need
  // p; in general it bounds them (rows before it that lack p are zeroed by the GEMM-1 epilogue).
  auto tile_rows_for = [&](int e, int i, int p) {
    const int r0 = i * BM, r1 = min(ne[e], r0 + BM);
    if (e >= E_res || p >= nsub_bits) return r1 - r0;
    int last = 0, off = 0;
    for (int sb = 0; sb < L.nsub; ++sb) {
      const int c = bin_count[e * L.nsub + sb];
      const int rev = L.nsub - 1 - sb;
      const bool has = (rev >> (nsub_bits - 1 - p)) & 1;
      if (has && c > 0 && off < r1 && off + c > r0) last = max(last, min(r1, off + c) - r0);
      off += c;
    }
    return last;
  };
  // Tall GEMM-1 items: when an expert's last row tile has at most kTallExtra rows, the item of the tile
  // before it (if that is full for the partition) computes them too, and the last tile gets no item of
  // its own: a few rows would otherwise pull the whole weight tile through another compute unit.
  auto absorbable = [&](int e, int i, int p) {
    if (i == 0) return false;
    if (i != tiles_of(ne[e]) - 1 || ne[e] - i * BM > kTallExtra) return false;
    if (!((tbits[ts[e] + i] >> p) & 1)) return false;
    return tile_rows_for(e, i - 1, p) == BM;
  };
  // Whether the batch gets them is decided by pricing both lists.  Items in 1/256 of a full one: a ragged
  // item of r rows 128 + r / 2 (half of every stage is its weight tile), a tall one 256 + 33 with up to 32
  // extra rows and 256 + 56 beyond (measured).  A list of N items of mean cost c is taken to last
  // ceil(N / units) * c, whole rounds of one item per compute unit: removing a tenth of the items is worth
  // a round or nothing, and the longer items of a list that still needs the same rounds make it slower.
  // est[]: items and summed cost of the list without / with tall items
  bool use_tall1 = L.tall_tiles == 2;
  const bool price_lists = lists1 && L.tall_tiles == 1 && (int64_t)T * L.K > BM;  // (no expert of a smaller batch has a second tile)
  if (price_lists) {
    // one thread per (expert, partition): the rows that need p are a prefix of the expert's rows (exactly so
    // with thresholds that grow with p; an estimate otherwise), so the group's items follow from one count
    int n0 = 0, w0 = 0, n1 = 0, w1 = 0;
    for (int gidx = tid; gidx < NG; gidx += kPlanThreads) {
      const int e = gidx / L.P, p = gidx % L.P;
      if (e >= E_res && p > 0) continue;
      int rows = ne[e];
      if (e < E_res && p < nsub_bits) {
        rows = 0;
        int off = 0;
        for (int sb = 0; sb < L.nsub; ++sb) {
          const int c = bin_count[e * L.nsub + sb];
          const int rev = L.nsub - 1 - sb;
          if (c > 0 && ((rev >> (nsub_bits - 1 - p)) & 1)) rows = off + c;
          off += c;
        }
      }
      if (rows == 0) continue;
      const int nt1 = e < E_res ? L.NT1 : L.NT1_sh;
      const int full = rows >> bm_sh, rem = rows & (BM - 1);
      const int n = full + (rem ? 1 : 0), w = full * 256 + (rem ? 128 + rem / 2 : 0);
      n0 += nt1 * n;
      w0 += nt1 * w;
      const int nt = tiles_of(ne[e]);
      if (nt >= 2 && ne[e] - (nt - 1) * BM <= kTallExtra && rows > (nt - 1) * BM) {  // the last tile's item goes into the one before
        n1 += nt1 * (n - 1);
        w1 += nt1 * (full * 256 + (rem <= 32 ? 33 : 56));
      } else {
        n1 += nt1 * n;
        w1 += nt1 * w;
      }
    }
    for (int o = 32; o > 0; o >>= 1) {
      n0 += __shfl_down(n0, o, 64);
      w0 += __shfl_down(w0, o, 64);
      n1 += __shfl_down(n1, o, 64);
      w1 += __shfl_down(w1, o, 64);
    }
    if ((tid & 63) == 0) {  // integer sums: the same in any order
      atomicAdd(&est[0], n0);
      atomicAdd(&est[1], w0);
      atomicAdd(&est[2], n1);
      atomicAdd(&est[3], w1);
    }
  }
  auto absorbed = [&](int e, int i, int p) { return use_tall1 && absorbable(e, i, p); };
  // 5. GEMM-2 items: every tile x every output column tile.  The compute units take the items in
  //    list order, one each.  Where that leaves units idle, items are split along K: every extra K
  //    range is an item of its own that writes a partial-output tile into a pool, and the combine
  //    kernel adds those tiles to the item's rows of Yp in a fixed order.
  //    (a) few row tiles (decode-sized batches): fewer items than units, each streaming a whole
  //        column tile of W2 alone -> all items are split, into as many ranges as keep the list
  //        within one item per unit;
  //    (b) the last round of a longer list is only partly full -> its items are split where the shorter
  //        pieces fill the units better (see below).
  //    A short last tile of an expert (at most kTallExtra rows) has no items of its own: the items of the
  //    tile before it are tall and compute its rows too (as in GEMM-1; here for all partitions at once).
  //    Only if the short tile keeps no partition that the tile before it drops: the tall items run over the
  //    partitions of the full tile, and where the short tile lacks one of them its rows of H are zeros
  //    (written by the GEMM-1 item of the full tile, see step 7).
  for (int i = tid; i < E_tot; i += kPlanThreads) {
    const int e = has_sh ? (i == 0 ? E_res : i - 1) : i;
    const int nt = tiles_of(ne[e]);
    int s = 0;
    if (L.tall_tiles && nt >= 2 && ne[e] - (nt - 1) * BM <= kTallExtra) s = (tbits[ts[e] + nt - 1] & ~tbits[ts[e] + nt - 2]) == 0 ? 1 : 0;
    abp[i] = s;
  }
  __shared__ int first_split_tile;  // first row tile (in row order) that has a split item: the combine kernel looks no tile before it up
  if (tid == 0) {
    abp[E_tot] = 0;
    first_split_tile = total_tiles;
  }
  __syncthreads();  // the sums of the pricing pass are complete too
  if (price_lists) {
    const int units = max(L.split_items, 1);
    const float t0 = est[0] > 0 ? (float)((est[0] + units - 1) / units) * (float)est[1] / (float)est[0] : 0.f;
    const float t1 = est[2] > 0 ? (float)((est[2] + units - 1) / units) * (float)est[3] / (float)est[2] : 0.f;
    use_tall1 = est[2] < est[0] && t1 <= t0;
  }
  const int total_short = block_excl_scan(abp, E_tot + 1, tmp);  // abp[E_tot] = total
  auto short_last = [&](int e) {  // read back from the scanned flags
    const int pos = has_sh ? (e == E_res ? 0 : e + 1) : e;
    return abp[pos + 1] - abp[pos];
  };
  if (lists2) {
    const int W2n = (total_tiles - total_short) * L.ND2;
    int nsplit = 1, first_split = W2n;  // items first_split .. W2n-1 (in list order) are split nsplit ways
    if (L.split_items > 0 && W2n > 0) {
      int ksp = L.Fp / kBK;
      if (has_sh) ksp = min(ksp, L.F_shT / kBK);
      if (W2n * 2 <= L.split_items) {
        while (nsplit < kMaxSplit && W2n * nsplit * 2 <= L.split_items && nsplit * 2 <= ksp) nsplit *= 2;
        first_split = 0;
      } else {
        // The last round holds `rest` items for split_items compute units.  Cut n ways they are rest * n
        // shorter items, which take ceil(rest * n / units) turns of 1/n of a round each (plus a fill and a
        // write-out per piece, worth about eight K stages): 192 items cut in four are three turns of a
        // quarter instead of a whole round at three quarters of the units.  The cheapest n that the pool
        // of partial tiles can hold wins; n = 1 (cost: one round) if none is cheaper.
        const int rest = W2n % L.split_items;
        if (rest > 0) {
          float best = 1.0f;
          const int item_stages = E_res > 0 ? L.P * (L.Fp / kBK) : L.F_shT / kBK;  // K stages of a long item
          const float piece = 8.0f / (float)max(item_stages, 1);                  // per-piece overhead in units of such an item
          for (int n = 2; n <= kMaxTailSplit && n <= ksp; ++n) {
            if (rest * (n - 1) > L.pool_tiles) break;
            const int turns = (rest * n + L.split_items - 1) / L.split_items;
            const float cost = (float)turns * (1.0f / (float)n + piece);
            if (cost < best - 0.04f) {  // a clear gain only: every extra range costs a partial tile written and read
              best = cost;
              nsplit = n;
            }
          }
          if (nsplit > 1) first_split = W2n - rest;
        }
      }
      if (nsplit == 1) first_split = W2n;
    }
    int32_t* split_of = (int32_t*)(ws + L.o_split_of);
    for (int gj = tid; gj < total_tiles * L.ND2; gj += kPlanThreads) {
      const int g = gj / L.ND2, jd = gj % L.ND2;
      const int e = tile_expert(g);
      const int i = g - ts[e];
      const int ksp = (e < E_res ? L.Fp : L.F_shT) / kBK;
      const int nt_all = tiles_of(ne[e]), sl = short_last(e);
      if (sl && i == nt_all - 1) continue;         // the short last tile: computed by the items of the tile before
      const bool tall = sl && i == nt_all - 2;
      Item2 v;
      v.row0 = rs[e] + i * BM;
      v.nrows = min(ne[e] - i * BM, BM) + (tall ? ne[e] - (i + 1) * BM : 0);
      v.e = e;
      v.jd = jd;
      v.kmask = tbits[g] | (tall ? tbits[g + 1] : 0);
      // list order (expert, column tile, row tile) if g2_rows_inner: the row tiles that share one column
      // tile of W2 are adjacent, run at the same time on one XCD and fetch the weights once;
      // else (row tile, column tile)
      const int nt_e = nt_all - sl;                                         // tiles of the expert that have items
      const int ts_e = ts[e] - abp[has_sh ? (e == E_res ? 0 : e + 1) : e];  // and of the experts before it
      const int slot = L.g2_rows_inner ? ts_e * L.ND2 + jd * nt_e + i : (ts_e + i) * L.ND2 + jd;
      if (slot < first_split) {
        v.ks_lo = 0;
        v.ks_n = ksp;
        v.split = 0;
        items2[slot] = v;
        if (L.split_items > 0) {
          split_of[gj] = -1;
          if (tall) split_of[gj + L.ND2] = -1;
        }
      } else {
        const int q = slot - first_split;  // q-th split item: its extra ranges use pool tiles q*(nsplit-1) ..
        atomicMin(&first_split_tile, g);
        for (int sp = 0; sp < nsplit; ++sp) {
          v.ks_lo = ksp * sp / nsplit;  // (at most a few thousand stages times 8)
          v.ks_n = ksp * (sp + 1) / nsplit - v.ks_lo;
          v.split = sp == 0 ? 0 : 1 + q * (nsplit - 1) + (sp - 1);
          items2[first_split + q * nsplit + sp] = v;
        }
        split_of[gj] = q * (nsplit - 1);
        if (tall) split_of[gj + L.ND2] = q * (nsplit - 1) | kSplitRowsOffset;  // rows of the short tile: BM further down the pool tiles
      }
    }
    __syncthreads();  // first_split_tile is final
    if (tid == 0) {
      counters[1] = first_split + (W2n - first_split) * nsplit;
      counters[2] = total_tiles - total_short;  // row tiles that have GEMM-2 items
      counters[3] = nsplit;
      counters[4] = first_split_tile;
    }
    return;
  }
  // 6. per (expert, partition): rank of each active tile among the active tiles of its group
  if (total_tiles <= kPlanTilesLds) {
    // keep patterns in LDS: one thread per (tile, partition) counts the active tiles before its own
    for (int gidx = tid; gidx < NG; gidx += kPlanThreads) ga[gidx] = gb[gidx] = 0;  // groups without tiles
    __syncthreads();
    for (int q = tid; q < total_tiles * L.P; q += kPlanThreads) {
      const int p = q % L.P, g = q / L.P;
      const int e = tile_expert(g);
      int cnt = 0;
      for (int j = ts[e]; j < g; ++j) cnt += (tbits[j] >> p) & 1;
      const int act = ((tbits[g] >> p) & 1) && !absorbed(e, g - ts[e], p) ? 1 : 0;
      act_rank[(size_t)g * L.P + p] = act ? cnt : -1;
      if (g - ts[e] == tiles_of(ne[e]) - 1) {  // the expert's last tile closes the group
        ga[e * L.P + p] = cnt + act;
        gb[e * L.P + p] = (cnt + act) * (e < E_res ? L.NT1 : L.NT1_sh);
      }
    }
  } else {  // very many tiles: one thread walks the tiles of a group
    for (int gidx = tid; gidx < NG; gidx += kPlanThreads) {
      int e = gidx / L.P, p = gidx % L.P;
      int nt = tiles_of(ne[e]);
      int cnt = 0;
      for (int i = 0; i < nt; ++i) {
        bool act = ((tbits[ts[e] + i] >> p) & 1) && !absorbed(e, i, p);
        act_rank[(size_t)(ts[e] + i) * L.P + p] = act ? cnt : -1;
        cnt += act ? 1 : 0;
      }
      ga[gidx] = cnt;
      gb[gidx] = cnt * (e < E_res ? L.NT1 : L.NT1_sh);
    }
  }
  __syncthreads();
  int total1 = block_excl_scan(gb, NG, tmp);
  // 7. GEMM-1 items in the order (expert, partition, neuron tile, row tile): the row tiles that
  //    share one weight tile are adjacent.  1 to 8 threads per (row tile, partition): each looks
  //    the tile up and writes the items of every S-th neuron tile.
  //    In the weight-streaming regime (few rows per expert) every item lasts as long as its weight
  //    tile takes to arrive, so the kernel lasts a whole number of rounds of one item per compute
  //    unit: when the last round is at most half full, its items are cut into halves of 64
  //    neurons, which fill it (an item of more than 128 rows, or of a last neuron tile of at most
  //    64 neurons, stays whole).
  int first_half = total1;  // list positions >= first_half belong to that last round
  if (may_halve_items1(L, T)) {
    const int rest = total1 % L.split_items;
    if (rest > 0 && rest * 2 <= L.split_items) first_half = total1 - rest;
  }
  const int nt1_max = has_sh && L.NT1_sh > L.NT1 ? L.NT1_sh : L.NT1;
  // threads that share the neuron tiles of one (row tile, partition): as many as would otherwise idle
  int S = kPlanThreads / max(total_tiles * L.P, 1);
  S = S < 1 ? 1 : S > 8 ? 8 : S;
  S = S > nt1_max ? nt1_max : S;
  for (int qs = tid; qs < total_tiles * L.P * S; qs += kPlanThreads) {
    const int part = qs % S, q = qs / S;
    const int p = q % L.P, g = q / L.P;
    const int rk = act_rank[(size_t)g * L.P + p];
    if (rk < 0) continue;
    const int e = tile_expert(g);
    const int nt1 = e < E_res ? L.NT1 : L.NT1_sh;
    const int gi = e * L.P + p;
    const int i = g - ts[e];
    Item1 v;
    v.row0 = rs[e] + i * BM;
    v.nfill = min(ne[e] - i * BM, BM);
    v.nrows = tile_rows_for(e, i, p);
    if (absorbed(e, i + 1, p)) {  // a tall item: the rows of the expert's short last tile follow directly
      v.nrows += tile_rows_for(e, i + 1, p);
      v.nfill += ne[e] - (i + 1) * BM;
    } else if (i + 2 == tiles_of(ne[e]) && short_last(e) && !((tbits[g + 1] >> p) & 1)) {
      // the tall GEMM-2 items of this tile multiply partition p over the short last tile's rows too, none
      // of which keeps it: their part of H is zeros, written by this item
      v.nfill += ne[e] - (i + 1) * BM;
    }
    v.e = e;
    v.p = p;
    v.pad = 0;
    for (int jt = part; jt < nt1; jt += S) {
      v.jt = jt;
      // MFMA path, at most 128 rows, a last neuron tile of at most 64 neurons: the half-tile variant of
      // the kernel takes it as a first half without a second one (half the weight bytes)
      const int live = (e < E_res ? L.Fp : L.F_shT) - jt * kMfmaNeur;
      v.half = L.split_items > 0 && v.nrows <= kMfmaBM / 2 && live <= kMfmaNeur / 2 ? 1 : 0;
      items1[gb[gi] + jt * ga[gi] + rk] = v;
    }
  }
  int total_slots = total1;
  if (first_half < total1) {  // the same for every thread
    // cut the items of the last round in two where that is possible (at most 128 rows, both halves
    // of the neuron tile exist); the list stays dense: item i moves up by the cuts before it
    __shared__ int slots_wave0, slots_all;
    __syncthreads();  // the items above are written
    const int rest = total1 - first_half;  // <= 128: wavefronts 0 and 1
    Item1 mine;
    int slots = 0;
    if (tid < rest) {
      mine = items1[first_half + tid];
      const int live = (mine.e < E_res ? L.Fp : L.F_shT) - mine.jt * kMfmaNeur;
      slots = mine.nrows <= kMfmaBM / 2 && live > kMfmaNeur / 2 ? 2 : 1;
    }
    int incl = slots;
    for (int o = 1; o < 64; o <<= 1) {
      const int up = __shfl_up(incl, o, 64);
      if ((tid & 63) >= o) incl += up;
    }
    if (tid == 63) slots_wave0 = incl;
    __syncthreads();  // and every item of the tail has been read before any is moved
    if (tid < rest) {
      const int at = first_half + incl - slots + (tid >= 64 ? slots_wave0 : 0);
      if (slots == 2) {
        mine.half = 1;
        items1[at] = mine;
        mine.half = 2;
        items1[at + 1] = mine;
      } else {
        items1[at] = mine;
      }
      if (tid == rest - 1) slots_all = at + slots;
    }
    __syncthreads();
    total_slots = slots_all;
  }
  if (tid == 0) counters[0] = total_slots;
}

hipError_t launch_plan(const Layout& L, int T, char* ws, hipStream_t s) {
  const int E_tot = L.E_res + (L.n_shared > 0 ? 1 : 0);
  const int NG = E_tot * L.P;
  size_t sh = sizeof(int32_t) * (size_t)(L.nbins + 5 * (E_tot + 2) + 2 * (NG + 1) + kPlanThreads + kPlanTilesLds + 8);
  if (sh > 48 * 1024) {  // hundreds of experts x 8 parts: up to ~78 KB, above what a launch gets without asking
    static PerDeviceOnce once;
    hipError_t e = once.run([] { return hipFuncSetAttribute((const void*)plan_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 104 * 1024); });
    if (e != hipSuccess) return e;
  }
  plan_kernel<<<dim3(2), dim3(kPlanThreads), sh, s>>>(L, T, ws);  // workgroup 0: GEMM-2 list, workgroup 1: GEMM-1 list
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------- scatter
// Places every pair with at least one kept unit into its bin's row range.  The order inside a bin
// is arbitrary (it is decided by atomics); the layer output does not depend on it because every
// row is computed independently of its tile neighbours.
constexpr int kScatterThreads = 256;
// PPT pairs per thread (pair u of a thread is block base + u * 256 + thread: coalesced).  A block
// claims its rows with one global atomic per bin it fills, so larger blocks mean fewer of those
// (with 256 bins and 256 pairs per block they were the whole cost on the fine-grained layers).
template <int PPT>
__global__ __launch_bounds__(kScatterThreads) void scatter_kernel(Layout L, int T, char* ws) {
  extern __shared__ int32_t lh[];  // [nbins]
  const int32_t* idx = (const int32_t*)(ws + L.o_idx);
  const uint8_t* keep = (const uint8_t*)(ws + L.o_keep);
  int32_t* cursor = (int32_t*)(ws + L.o_cursor);
  int32_t* pair_row = (int32_t*)(ws + L.o_pair_row);
  int32_t* row_token = (int32_t*)(ws + L.o_row_token);
  uint8_t* row_bits = (uint8_t*)(ws + L.o_row_bits);
  const int nsub_bits = L.P < kSubBits ? L.P : kSubBits;
  const int64_t npairs = (int64_t)T * L.K;
  const int64_t pr0 = (int64_t)blockIdx.x * (kScatterThreads * PPT) + threadIdx.x;
  for (int i = threadIdx.x; i < L.nbins; i += kScatterThreads) lh[i] = 0;
  int bits[PPT], ex[PPT], bin[PPT], rank[PPT];
#pragma unroll
  for (int u = 0; u < PPT; ++u) {
    const int64_t pr = pr0 + u * kScatterThreads;
    bits[u] = pr < npairs ? keep[pr] : 0;
    ex[u] = pr < npairs ? idx[pr] : 0;
  }
  __syncthreads();
#pragma unroll
  for (int u = 0; u < PPT; ++u) {
    bin[u] = -1;
    rank[u] = 0;
    if (bits[u]) {
      bin[u] = (ex[u] - L.lo) * L.nsub + sub_of_bits(bits[u], nsub_bits);
      rank[u] = atomicAdd(&lh[bin[u]], 1);
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < L.nbins; i += kScatterThreads) {
    int c = lh[i];
    if (c) lh[i] = atomicAdd(&cursor[i], c);
  }
  __syncthreads();
#pragma unroll
  for (int u = 0; u < PPT; ++u) {
    const int64_t pr = pr0 + u * kScatterThreads;
    if (pr < npairs) {
      int row = -1;
      if (bin[u] >= 0) {
        row = lh[bin[u]] + rank[u];
        row_token[row] = (int32_t)(pr / L.K);
        row_bits[row] = (uint8_t)bits[u];
      }
      pair_row[pr] = row;
    }
    // the shared pseudo-expert's rows are the tokens themselves, at the start of the row space
    if (L.n_shared > 0 && pr < T) {
      row_token[pr] = (int32_t)pr;
      row_bits[pr] = 1;
    }
  }
}

hipError_t launch_scatter(const Layout& L, int T, char* ws, hipStream_t s) {
  int64_t n = (int64_t)T * L.K;
  if (n <= 0) return hipSuccess;
  size_t sh = sizeof(int32_t) * (size_t)(L.nbins > 0 ? L.nbins : 1);
  // as many pairs per thread as leave about 64 blocks or more
  const int64_t per = n / (64 * kScatterThreads);
  auto blocks = [&](int ppt) { return dim3((unsigned)((n + (int64_t)kScatterThreads * ppt - 1) / ((int64_t)kScatterThreads * ppt))); };
  if (per >= 8) scatter_kernel<8><<<blocks(8), dim3(kScatterThreads), sh, s>>>(L, T, ws);
  else if (per >= 4) scatter_kernel<4><<<blocks(4), dim3(kScatterThreads), sh, s>>>(L, T, ws);
  else if (per >= 2) scatter_kernel<2><<<blocks(2), dim3(kScatterThreads), sh, s>>>(L, T, ws);
  else scatter_kernel<1><<<blocks(1), dim3(kScatterThreads), sh, s>>>(L, T, ws);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------- combine
// y[t] = sum_k g[t][k] * Yp[row(t,k)] (+ Yp[shared row t]); Eq. 3 restricted to the kept units.
// One writer per output element, slots added in slot order: no atomics.
// Partial outputs still carry the powers of two of the packed weights; w2_inv = 2^-(s+k) takes them
// out here (exact, so the result is the one unscaled weights would give; 1 on the generic path).
// They are fp32, or (HALF) half precision times kYpHalfScale, which is taken out here as well.
// 16 bytes of partial outputs: VEC = 4 floats, or 8 half-precision values.  The rows of a token are
// loaded as raw 16-byte vectors (all in flight together) and widened one row at a time, so that the
// kernel stays within the registers of full occupancy.
template <bool HALF>
struct Partials {
  static constexpr int VEC = HALF ? 8 : 4;
  static __device__ __forceinline__ uint4 load(const char* base, size_t idx) { return *(const uint4*)(base + idx * (HALF ? 2 : 4)); }
  static __device__ __forceinline__ void widen(const uint4& r, float (&v)[VEC]) {
    if constexpr (HALF) {
      typedef _Float16 h8 __attribute__((ext_vector_type(8)));
      const h8 h = __builtin_bit_cast(h8, r);
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = (float)h[i];
    } else {
      v[0] = __uint_as_float(r.x), v[1] = __uint_as_float(r.y), v[2] = __uint_as_float(r.z), v[3] = __uint_as_float(r.w);
    }
  }
};

template <typename OutT, int KB, bool HALF>
__global__ __launch_bounds__(256) void combine_kernel(Layout L, int T, const char* ws, OutT* y, const float* w2_inv_p) {
  using PT = Partials<HALF>;
  constexpr int VEC = PT::VEC;  // columns per thread (D % 8 == 0 where HALF is used: the matrix-core path)
  const float w2_inv = (w2_inv_p ? *w2_inv_p : 1.f) * (HALF ? 1.0f / kYpHalfScale : 1.f);
  const char* Yp = ws + L.o_Yp;
  const float* w = (const float*)(ws + L.o_w);
  const int32_t* pair_row = (const int32_t*)(ws + L.o_pair_row);
  const int DV = L.D / VEC;
  const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (q >= (int64_t)T * DV) return;
  const int t = (int)(q / DV);
  const int d = (int)(q % DV) * VEC;
  // all row indices first, then all row loads in flight together, then the sum in slot order
  int row[KB];
  float g[KB];
#pragma unroll
  for (int k = 0; k < KB; ++k) {
    row[k] = k < L.K ? pair_row[(size_t)t * L.K + k] : -1;
    g[k] = k < L.K ? w[(size_t)t * L.K + k] * w2_inv : 0.f;
  }
  uint4 raw[KB];
#pragma unroll
  for (int k = 0; k < KB; ++k) raw[k] = row[k] >= 0 ? PT::load(Yp, (size_t)row[k] * L.D + d) : make_uint4(0, 0, 0, 0);
  float acc[VEC];
#pragma unroll
  for (int i = 0; i < VEC; ++i) acc[i] = 0.f;
  const int32_t* counters = (const int32_t*)(ws + L.o_counters);
  const int nsplit = counters[3];
  const int split_row0 = counters[4] * L.BM;  // rows before it belong to tiles without split items
  const int32_t* split_of = (const int32_t*)(ws + L.o_split_of);
  const char* pool = ws + L.o_pool;
  const int jd = d / kMfmaBN2, dc = d - jd * kMfmaBN2;
  // GEMM-2 split K: the partial-output tiles of the extra K ranges of row r are added in range order
  auto add_extra = [&](int r, float (&into)[VEC]) {
    const int tile = r / L.BM;
    int first = split_of[(size_t)tile * L.ND2 + jd];
    if (first < 0) return;
    const int rofs = first & kSplitRowsOffset ? L.BM : 0;  // a short last tile: its rows follow those of the tile before
    first &= ~kSplitRowsOffset;
    size_t src = ((size_t)first * kPoolRows + (r - tile * L.BM) + rofs) * kMfmaBN2 + dc;
    for (int sp = 1; sp < nsplit; ++sp) {
      float u[VEC];
      PT::widen(PT::load(pool, src), u);
#pragma unroll
      for (int i = 0; i < VEC; ++i) into[i] += u[i];
      src += (size_t)kPoolRows * kMfmaBN2;
    }
  };
  if (L.n_shared > 0) {  // the shared experts' rows sit first in the row space (weight 1)
    PT::widen(PT::load(Yp, (size_t)t * L.D + d), acc);
    if (nsplit > 1 && t >= split_row0) add_extra(t, acc);
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] *= w2_inv;
  }
#pragma unroll
  for (int k = 0; k < KB; ++k) {
    if (row[k] >= 0) {
      float v[VEC];
      PT::widen(raw[k], v);
      if (nsplit > 1 && row[k] >= split_row0) add_extra(row[k], v);
#pragma unroll
      for (int i = 0; i < VEC; ++i) acc[i] += g[k] * v[i];
    }
  }
  if constexpr (sizeof(OutT) == 4) {
    float* dst = (float*)y + (size_t)t * L.D + d;
#pragma unroll
    for (int i = 0; i < VEC; i += 4) *(float4*)(dst + i) = make_float4(acc[i], acc[i + 1], acc[i + 2], acc[i + 3]);
  } else {
    uint16_t* dst = (uint16_t*)y + (size_t)t * L.D + d;
    uint16_t o[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) o[i] = f32_to_bf16(acc[i]);
    if constexpr (VEC == 8) {
      *(uint4*)dst = make_uint4(o[0] | ((uint32_t)o[1] << 16), o[2] | ((uint32_t)o[3] << 16), o[4] | ((uint32_t)o[5] << 16),
                                o[6] | ((uint32_t)o[7] << 16));
    } else {
      *(uint2*)dst = make_uint2(o[0] | ((uint32_t)o[1] << 16), o[2] | ((uint32_t)o[3] << 16));
    }
  }
}

// any D (no vector access): one thread per output element
template <typename OutT>
__global__ __launch_bounds__(256) void combine_scalar_kernel(Layout L, int T, const char* ws, OutT* y) {
  const float* Yp = (const float*)(ws + L.o_Yp);
  const float* w = (const float*)(ws + L.o_w);
  const int32_t* pair_row = (const int32_t*)(ws + L.o_pair_row);
  const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (q >= (int64_t)T * L.D) return;
  const int t = (int)(q / L.D);
  const int d = (int)(q % L.D);
  float acc = 0.f;
  for (int k = 0; k < L.K; ++k) {
    int row = pair_row[(size_t)t * L.K + k];
    if (row >= 0) acc += w[(size_t)t * L.K + k] * Yp[(size_t)row * L.D + d];
  }
  if (L.n_shared > 0) acc += Yp[(size_t)t * L.D + d];
  if constexpr (sizeof(OutT) == 4) ((float*)y)[q] = acc;
  else ((uint16_t*)y)[q] = f32_to_bf16(acc);
}

hipError_t launch_combine(const Layout& L, int T, const char* packed, char* ws, void* y, hipStream_t s) {
  if (T <= 0) return hipSuccess;
  const float* w2_inv = L.mfma ? (const float*)(packed + L.p_scale) + 2 : nullptr;
  if (L.D % 4 == 0) {
    int64_t n = (int64_t)T * (L.D / (L.yp_half ? 8 : 4));
    dim3 grid((unsigned)((n + 255) / 256)), block(256);
#define DSMOE_COMBINE(KB)                                                                      \
  do {                                                                                          \
    if (L.yp_half) {                                                                              \
      if (L.y_f32) combine_kernel<float, KB, true><<<grid, block, 0, s>>>(L, T, ws, (float*)y, w2_inv); \
      else combine_kernel<uint16_t, KB, true><<<grid, block, 0, s>>>(L, T, ws, (uint16_t*)y, w2_inv);  \
    } else {                                                                                      \
      if (L.y_f32) combine_kernel<float, KB, false><<<grid, block, 0, s>>>(L, T, ws, (float*)y, w2_inv); \
      else combine_kernel<uint16_t, KB, false><<<grid, block, 0, s>>>(L, T, ws, (uint16_t*)y, w2_inv);  \
    }                                                                                             \
  } while (0)
    if (L.K <= 2) DSMOE_COMBINE(2);
    else if (L.K <= 4) DSMOE_COMBINE(4);
    else if (L.K <= 8) DSMOE_COMBINE(8);
    else DSMOE_COMBINE(16);
#undef DSMOE_COMBINE
  } else {
    int64_t n = (int64_t)T * L.D;
    dim3 grid((unsigned)((n + 255) / 256)), block(256);
    if (L.y_f32) combine_scalar_kernel<float><<<grid, block, 0, s>>>(L, T, ws, (float*)y);
    else combine_scalar_kernel<uint16_t><<<grid, block, 0, s>>>(L, T, ws, (uint16_t*)y);
  }
  return hipGetLastError();
}

}  // namespace dsmoe
