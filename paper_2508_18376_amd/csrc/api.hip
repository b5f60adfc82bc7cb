// C ABI of libdsmoe (see include/dsmoe.h): argument checks, workspace / packed-buffer layout and
// the kernel sequence of each entry point.  No device memory is allocated here.
#include <stdlib.h>
#include <string.h>

#include <new>

#include "common.h"

using namespace dsmoe;

namespace {

inline int64_t align_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }
inline int cdiv(int a, int b) { return (a + b - 1) / b; }

bool build_layout(const dsmoe_config& c, Layout& L) {
  memset(&L, 0, sizeof(L));
  if (c.d_model < 1 || c.d_ff < 1) return false;
  if (c.n_experts < 1 || c.n_experts > kMaxExperts) return false;
  if (c.top_k < 1 || c.top_k > c.n_experts || c.top_k > kMaxTopK) return false;
  if (c.n_part < 1 || c.n_part > kMaxPart || c.d_ff % c.n_part != 0) return false;
  if (c.n_shared < 0 || (c.n_shared > 0 && c.d_ff_shared < 1)) return false;
  if (c.expert_lo < 0 || c.expert_hi > c.n_experts || c.expert_lo >= c.expert_hi) return false;
  if (c.max_tokens < 1) return false;
  if (c.dtype != DSMOE_F32 && c.dtype != DSMOE_BF16) return false;
  if (c.renorm_combine != 0 && c.renorm_combine != 1) return false;
  if (c.y_fp32 != 0 && c.y_fp32 != 1) return false;
  if (c.h_scale_log2 < -40 || c.h_scale_log2 > 40) return false;
  if (c.partial_fp32 != 0 && c.partial_fp32 != 1) return false;
  if (c.tall_items < -1 || c.tall_items > 1) return false;
  if ((int64_t)c.max_tokens * c.top_k * c.n_part > (int64_t)1 << 30) return false;
  if ((int64_t)c.n_shared * c.d_ff_shared > (int64_t)1 << 30) return false;

  L.D = c.d_model;
  L.F = c.d_ff;
  L.E = c.n_experts;
  L.K = c.top_k;
  L.P = c.n_part;
  L.Fp = c.d_ff / c.n_part;
  L.lo = c.expert_lo;
  L.hi = c.expert_hi;
  L.E_res = c.expert_hi - c.expert_lo;
  L.n_shared = c.n_shared;
  L.F_shT = c.n_shared * c.d_ff_shared;
  L.renorm = c.renorm_combine;
  L.dtype = c.dtype;
  L.y_f32 = (c.dtype == DSMOE_F32 || c.y_fp32) ? 1 : 0;
  L.max_tokens = c.max_tokens;

  L.mfma = (c.dtype == DSMOE_BF16 && L.D % kBK == 0 && L.Fp % kBK == 0 && (L.n_shared == 0 || L.F_shT % kBK == 0) &&
            (int64_t)c.max_tokens * L.D * 2 < ((int64_t)1 << 31))
               ? 1
               : 0;
  L.yp_half = (L.mfma && !c.partial_fp32) ? 1 : 0;
  L.h_shift = L.mfma ? c.h_scale_log2 : 0;  // the generic path keeps the activation in fp32: nothing to scale
  const int64_t elem = c.dtype == DSMOE_F32 ? 4 : 2;
  L.BM = L.mfma ? kMfmaBM : kGenBM;
  const int neur = L.mfma ? kMfmaNeur : kGenBN;
  const int bn2 = L.mfma ? kMfmaBN2 : kGenBN;
  L.NT1 = cdiv(L.Fp, neur);
  L.NT1_sh = L.n_shared > 0 ? cdiv(L.F_shT, neur) : 0;
  L.ND2 = cdiv(L.D, bn2);
  L.split_items = L.mfma ? kSplitItems : 0;
  // GEMM-2 item order.  Long contractions (a 256-column tile of W2 of 1 MiB or more) do not stay in an
  // XCD's L2 from one row tile to the next: the row tiles that share a column tile are then made
  // adjacent so they stream it together (measured: -9 % on d_ff 14336, +7 % on d_ff 1024..1408).
  L.g2_rows_inner = (int64_t)L.F * kMfmaBN2 * 2 >= (1 << 20) ? 1 : 0;
  // tall items need whole neuron tiles (the variant for a half-full last neuron tile has no tall form)
  auto whole_tiles = [](int n) { const int m = n % kMfmaNeur; return m == 0 || m > kMfmaNeur / 2; };
  L.tall_tiles = L.mfma && c.tall_items >= 0 && whole_tiles(L.Fp) && (L.n_shared == 0 || whole_tiles(L.F_shT)) ? 1 + c.tall_items : 0;
  const int nsub_bits = L.P < kSubBits ? L.P : kSubBits;
  L.nsub = 1 << nsub_bits;
  L.nbins = L.E_res * L.nsub;
  const int Tm = c.max_tokens;
  L.sh_rows = L.n_shared > 0 ? (int)align_up(Tm, L.BM) : 0;
  const int rt = routed_tiles_bound(L, Tm);
  L.row_cap = L.sh_rows + rt * L.BM;
  L.max_tiles = rt + shared_tiles(L, Tm);
  L.max_items1 = items1_whole_bound(L, Tm) + L.split_items / 2;  // a smaller batch may cut its last items in two
  // partial-output tiles the K splits of GEMM-2 can need: contexts whose largest batch has so few row
  // tiles that every item is split (decode sizes) stay within one extra tile per compute unit
  L.pool_tiles = L.split_items == 0 ? 0 : ((int64_t)L.max_tiles * L.ND2 * 2 <= L.split_items ? kSplitItems : kPoolTiles);
  L.max_items2 = L.max_tiles * L.ND2 + L.pool_tiles;

  int64_t o = 0;
  auto take = [&](int64_t bytes) {
    int64_t at = o;
    o = align_up(o + bytes, 256);
    return at;
  };
  const int64_t npairs = (int64_t)Tm * L.K;
  L.o_idx = take(npairs * 4);
  L.o_w = take(npairs * 4);
  L.o_keep = take(npairs);
  L.o_pair_row = take(npairs * 4);
  {  // one histogram row per route block
    const int rows_small = cdiv(Tm < kWaveSmallBatch ? Tm : kWaveSmallBatch, kWaveBlockTokens), rows_big = cdiv(Tm, kRouteBlockTokens);
    L.o_bin_count = take((int64_t)(rows_small > rows_big ? rows_small : rows_big) * L.nbins * 4);
  }
  L.o_cursor = take((int64_t)L.nbins * 4);
  L.o_exp_nrows = take((int64_t)L.E_res * 4);
  L.o_exp_row0 = take((int64_t)L.E_res * 4);
  L.o_counters = take(32);
  L.o_tile_bits = take((int64_t)L.max_tiles * 4);
  L.o_act_rank = take((int64_t)L.max_tiles * L.P * 4);
  L.o_items1 = take((int64_t)L.max_items1 * sizeof(Item1));
  L.o_items2 = take((int64_t)L.max_items2 * sizeof(Item2));
  L.o_row_token = take((int64_t)L.row_cap * 4);
  L.o_row_bits = take((int64_t)L.row_cap);
  auto take_big = [&](int64_t bytes) {  // the large arrays start on 2 MiB boundaries
    o = align_up(o, 2 << 20);
    return take(bytes);
  };
  const int64_t helem = L.mfma ? 2 : 4;  // H: half precision on the MFMA path, fp32 on the generic path
  L.o_H = take_big((int64_t)(L.row_cap - L.sh_rows) * L.F * helem);
  L.o_Hs = take_big((int64_t)L.sh_rows * L.F_shT * helem);
  L.o_Yp = take_big((int64_t)L.row_cap * L.D * (L.yp_half ? 2 : 4));
  L.o_tau0 = take((int64_t)L.E * L.P * 4);
  L.o_sel = take((int64_t)(L.E + 1) * (kSelBins + 2) * 4);  // directly behind tau0: one fill clears both; row E: resident pairs
  L.o_logits = take((int64_t)Tm * L.E * 4);
  L.o_perm_check = take(((int64_t)L.E_res * L.F + 1) * 4);
  L.o_pool = take_big((int64_t)L.pool_tiles * kPoolRows * kMfmaBN2 * (L.yp_half ? 2 : 4));  // partial outputs of split K ranges
  L.o_split_of = take(L.split_items > 0 ? (int64_t)L.max_tiles * L.ND2 * 4 : 0);          // (row tile, column tile) -> first pool tile, or -1
  L.ws_bytes = o;

  // packed weights
  int64_t q = 0;
  auto takep = [&](int64_t bytes) {
    int64_t at = q;
    q = align_up(q + bytes, 256);
    return at;
  };
  if (L.mfma) {
    const int64_t KS1 = L.D / kBK;
    L.w13_expert_bytes = (int64_t)L.P * L.NT1 * KS1 * kStageBytes;
    L.w2_expert_bytes = (int64_t)L.ND2 * (L.F / kBK) * kStageBytes;
    L.p_w13 = takep(L.w13_expert_bytes * L.E_res);
    L.p_w2 = takep(L.w2_expert_bytes * L.E_res);
    L.p_sw13 = takep((int64_t)L.NT1_sh * KS1 * kStageBytes);
    L.p_sw2 = takep(L.n_shared > 0 ? (int64_t)L.ND2 * (L.F_shT / kBK) * kStageBytes : 0);
    L.p_scale = takep(16);
  } else {
    L.w13_expert_bytes = (int64_t)L.D * L.F * elem;
    L.w2_expert_bytes = (int64_t)L.F * L.D * elem;
    L.p_w13 = takep(2 * L.w13_expert_bytes * L.E_res);
    L.p_w2 = takep(L.w2_expert_bytes * L.E_res);
    L.p_sw13 = takep(2 * (int64_t)L.D * L.F_shT * elem);
    L.p_sw2 = takep((int64_t)L.F_shT * L.D * elem);
  }
  // the permutation check borrows the start of the packed buffer for its counters
  const int64_t need_check = ((int64_t)L.E_res * L.F + 1) * 4;
  if (q < need_check) q = align_up(need_check, 256);
  L.packed_bytes = q;
  L.router_mfma = (c.dtype == DSMOE_BF16 && L.D % 64 == 0) ? 1 : 0;
  L.router_bytes = L.router_mfma ? (int64_t)L.D * ((L.E + 31) / 32 * 32) * 2 : (int64_t)L.D * L.E * 4;
  return true;
}

inline int hip_fail(Ctx* ctx, hipError_t e) {
  ctx->last_hip = (int)e;
  return DSMOE_EHIP;
}

// Workspace of moe_dualsparse_forward_static: device memory that belongs to the loaded library, one
// copy per GPU, held until the process ends.  In host code the array's name only stands for the
// symbol; the device address of the current GPU's copy comes from hipGetSymbolAddress and is kept
// per device in g_scratch_ptr.  Nothing in it has to start at zero: every kernel of the layer
// writes what a later one reads.
static __device__ __align__(256) unsigned char scratch[DSMOE_STATIC_SCRATCH_BYTES];
void* g_scratch_ptr[kMaxDevices] = {};
PerDeviceOnce g_scratch_once;

// device address of the current GPU's scratch array (looked up on the first call per device)
hipError_t static_scratch(void** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  e = g_scratch_once.run([dev] {
    void* p = nullptr;
    hipError_t e2 = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e2 == hipSuccess && p == nullptr) e2 = hipErrorInvalidSymbol;
    if (e2 == hipSuccess) g_scratch_ptr[dev] = p;
    return e2;
  });
  if (e != hipSuccess) return e;
  {
    std::lock_guard<std::mutex> g(g_scratch_once.mu);  // pairs with the write above
    *out = g_scratch_ptr[dev];
  }
  return hipSuccess;
}

}  // namespace

extern "C" {

int dsmoe_create(const dsmoe_config* cfg, dsmoe_ctx** out) {
  if (!cfg || !out) return DSMOE_EINVAL;
  *out = nullptr;
  Ctx* c = new (std::nothrow) Ctx();
  if (!c) return DSMOE_EINVAL;
  c->cfg = *cfg;
  c->last_hip = 0;
  c->last_sh_rows = 0;
  if (!build_layout(*cfg, c->L)) {
    delete c;
    return DSMOE_EINVAL;
  }
  *out = reinterpret_cast<dsmoe_ctx*>(c);
  return DSMOE_OK;
}

int dsmoe_destroy(dsmoe_ctx* ctx) {
  if (!ctx) return DSMOE_EINVAL;
  delete reinterpret_cast<Ctx*>(ctx);
  return DSMOE_OK;
}

size_t dsmoe_packed_bytes(const dsmoe_ctx* ctx) { return ctx ? (size_t) reinterpret_cast<const Ctx*>(ctx)->L.packed_bytes : 0; }
size_t dsmoe_router_packed_bytes(const dsmoe_ctx* ctx) { return ctx ? (size_t) reinterpret_cast<const Ctx*>(ctx)->L.router_bytes : 0; }
size_t dsmoe_workspace_bytes(const dsmoe_ctx* ctx) { return ctx ? (size_t) reinterpret_cast<const Ctx*>(ctx)->L.ws_bytes : 0; }
int dsmoe_last_hip_error(const dsmoe_ctx* ctx) { return ctx ? reinterpret_cast<const Ctx*>(ctx)->last_hip : 0; }
int dsmoe_uses_mfma(const dsmoe_ctx* ctx) { return ctx ? reinterpret_cast<const Ctx*>(ctx)->L.mfma : 0; }

const char* dsmoe_strerror(int status) {
  switch (status) {
    case DSMOE_OK: return "ok";
    case DSMOE_EINVAL: return "invalid argument (shape, divisibility, limit, null pointer or T > max_tokens)";
    case DSMOE_EPERM: return "perm is not a permutation of the expert's neurons";
    case DSMOE_ENOSPC: return "the batch needs more workspace than the library's static scratch array holds";
    case DSMOE_EHIP: return "HIP call or kernel launch failed";
    default: return "unknown dsmoe status";
  }
}

int moe_partition_weights(dsmoe_ctx* ctx_, const void* w1, const void* w3, const void* w2, const void* sh_w1,
                          const void* sh_w3, const void* sh_w2, const int32_t* perm, void* packed_out, void* stream) {
  Ctx* ctx = reinterpret_cast<Ctx*>(ctx_);
  if (!ctx || !w1 || !w3 || !w2 || !packed_out) return DSMOE_EINVAL;
  const Layout& L = ctx->L;
  if (L.n_shared > 0 && (!sh_w1 || !sh_w3 || !sh_w2)) return DSMOE_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  hipError_t err;
  if (perm) {
    int32_t* scratch = (int32_t*)packed_out;
    err = launch_perm_check(L, perm, scratch, s);
    if (err != hipSuccess) return hip_fail(ctx, err);
    int32_t bad = 0;
    err = hipMemcpyAsync(&bad, scratch + (size_t)L.E_res * L.F, sizeof(int32_t), hipMemcpyDeviceToHost, s);
    if (err != hipSuccess) return hip_fail(ctx, err);
    err = hipStreamSynchronize(s);
    if (err != hipSuccess) return hip_fail(ctx, err);
    if (bad != 0) return DSMOE_EPERM;
  }
  err = launch_pack(L, w1, w3, w2, sh_w1, sh_w3, sh_w2, perm, (char*)packed_out, ctx->cfg.n_shared, ctx->cfg.d_ff_shared, s);
  if (err != hipSuccess) return hip_fail(ctx, err);
  err = hipStreamSynchronize(s);
  if (err != hipSuccess) return hip_fail(ctx, err);
  return DSMOE_OK;
}

int moe_route_and_mask(dsmoe_ctx* ctx_, const float* logits, int32_t T, const float* tau, int32_t* topk_idx, float* topk_w,
                       uint8_t* keep_bits, int32_t* group_count, void* stream) {
  Ctx* ctx = reinterpret_cast<Ctx*>(ctx_);
  if (!ctx || T < 0 || !tau || !group_count) return DSMOE_EINVAL;
  if (T > 0 && (!logits || !topk_idx || !topk_w || !keep_bits)) return DSMOE_EINVAL;
  const Layout& L = ctx->L;
  if (T > L.max_tokens) return DSMOE_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  hipError_t err = launch_fill_i32(group_count, (int64_t)L.E * L.P, 0, s);
  if (err != hipSuccess) return hip_fail(ctx, err);
  err = launch_route(L, logits, T, tau, topk_idx, topk_w, keep_bits, nullptr, group_count, s);
  if (err != hipSuccess) return hip_fail(ctx, err);
  return DSMOE_OK;
}

// The layer's kernel sequence.  router_packed != nullptr: the logits are computed first (into
// logits_buf) from x and the packed gating weights; otherwise logits_buf holds the caller's logits.
static int forward_impl(Ctx* ctx, const Layout& base, const void* packed, const char* router_packed, const void* x,
                        const float* logits_buf, const float* tau, int32_t T, void* y, void* workspace, void* stream) {
  // The shared experts' rows come first in the row space and the routed rows start at the next
  // tile boundary after the T rows of THIS call (the plan kernel places them there), so the layout
  // every kernel of the call sees carries that boundary, not the one max_tokens would give.
  Layout L = base;
  L.sh_rows = L.n_shared > 0 ? (int)align_up(T, L.BM) : 0;
  ctx->last_sh_rows = L.sh_rows;
  const float* logits = logits_buf;
  if (T == 0) return DSMOE_OK;
  hipStream_t s = (hipStream_t)stream;
  char* ws = (char*)workspace;
  hipError_t err = hipSuccess;
  // optional per-kernel events (benchmarks only); the call stays asynchronous either way
  Profile& pf = ctx->prof;
  const bool rec = pf.level > 0 && pf.calls < pf.max_calls;
  const int per_call = pf.level == 2 ? kNumKernels + 1 : 2;
  hipEvent_t* ev = rec ? pf.ev + (size_t)pf.calls * per_call : nullptr;
  auto mark = [&](int boundary) {  // boundary b sits before kernel b (b = kNumKernels: after the last)
    if (!rec || err != hipSuccess) return;
    if (pf.level == 2) err = hipEventRecord(ev[boundary], s);
    else if (boundary == 4) err = hipEventRecord(ev[0], s);
    else if (boundary == 5) err = hipEventRecord(ev[1], s);
  };
#define DSMOE_STEP(b, call) \
  do {                      \
    mark(b);                \
    if (err == hipSuccess) err = (call); \
  } while (0)
  mark(0);
  if (router_packed && err == hipSuccess) err = launch_router(L, T, router_packed, x, const_cast<float*>(logits_buf), s);
  DSMOE_STEP(1, launch_route(L, logits, T, tau, (int32_t*)(ws + L.o_idx), (float*)(ws + L.o_w), (uint8_t*)(ws + L.o_keep),
                             (int32_t*)(ws + L.o_bin_count), nullptr, s));
  DSMOE_STEP(2, launch_plan(L, T, ws, s));
  DSMOE_STEP(3, launch_scatter(L, T, ws, s));
  DSMOE_STEP(4, L.mfma ? launch_gemm1_mfma(L, T, (const char*)packed, x, ws, 0, s)
                       : launch_gemm1_generic(L, T, (const char*)packed, x, ws, 0, s));
  DSMOE_STEP(5, L.mfma ? launch_gemm2_mfma(L, T, (const char*)packed, ws, s) : launch_gemm2_generic(L, T, (const char*)packed, ws, s));
  DSMOE_STEP(6, launch_combine(L, T, (const char*)packed, ws, y, s));
  mark(kNumKernels);
#undef DSMOE_STEP
  if (err != hipSuccess) return hip_fail(ctx, err);
  if (rec) pf.calls += 1;
  return DSMOE_OK;
}

int moe_dualsparse_forward(dsmoe_ctx* ctx_, const void* packed, const void* x, const float* logits, const float* tau,
                           int32_t T, void* y, void* workspace, void* stream) {
  Ctx* ctx = reinterpret_cast<Ctx*>(ctx_);
  if (!ctx || T < 0 || !packed || !tau || !workspace) return DSMOE_EINVAL;
  if (T > 0 && (!x || !logits || !y)) return DSMOE_EINVAL;
  if (((uintptr_t)workspace & 255) != 0 || ((uintptr_t)packed & 15) != 0) return DSMOE_EINVAL;
  if (T > ctx->L.max_tokens) return DSMOE_EINVAL;
  return forward_impl(ctx, ctx->L, packed, nullptr, x, logits, tau, T, y, workspace, stream);
}

int moe_dualsparse_forward_static(dsmoe_ctx* ctx_, const void* packed, const void* x, const float* logits, const float* tau,
                                  int32_t T, void* y, void* stream) {
  Ctx* ctx = reinterpret_cast<Ctx*>(ctx_);
  if (!ctx || T < 0 || !packed || !tau) return DSMOE_EINVAL;
  if (T > 0 && (!x || !logits || !y)) return DSMOE_EINVAL;
  if (((uintptr_t)packed & 15) != 0) return DSMOE_EINVAL;
  if (T > ctx->L.max_tokens) return DSMOE_EINVAL;
  // the workspace layout of a context made for exactly this batch: the offsets depend on T, so a
  // small batch of a large layer fits the array even if the context's own max_tokens would not
  dsmoe_config c = ctx->cfg;
  c.max_tokens = T > 0 ? T : 1;
  Layout L;
  if (!build_layout(c, L)) return DSMOE_EINVAL;
  // the packed weights were laid out for the context's own layout: the two must agree on the kernels
  if (L.mfma != ctx->L.mfma || L.packed_bytes != ctx->L.packed_bytes) return DSMOE_EINVAL;
  if (L.ws_bytes > (int64_t)DSMOE_STATIC_SCRATCH_BYTES) return DSMOE_ENOSPC;
  void* ws = nullptr;
  hipError_t e = static_scratch(&ws);
  if (e != hipSuccess) return hip_fail(ctx, e);
  return forward_impl(ctx, L, packed, nullptr, x, logits, tau, T, y, ws, stream);
}

size_t dsmoe_static_workspace_need(const dsmoe_ctx* ctx_, int32_t T) {
  const Ctx* ctx = reinterpret_cast<const Ctx*>(ctx_);
  if (!ctx || T < 0) return 0;
  dsmoe_config c = ctx->cfg;
  c.max_tokens = T > 0 ? T : 1;
  Layout L;
  if (!build_layout(c, L)) return 0;
  return (size_t)L.ws_bytes;
}

int moe_pack_router(dsmoe_ctx* ctx_, const void* wg, void* router_packed, void* stream) {
  Ctx* ctx = reinterpret_cast<Ctx*>(ctx_);
  if (!ctx || !wg || !router_packed || ((uintptr_t)router_packed & 15) != 0) return DSMOE_EINVAL;
  hipError_t err = launch_router_pack(ctx->L, wg, (char*)router_packed, (hipStream_t)stream);
  if (err != hipSuccess) return hip_fail(ctx, err);
  return DSMOE_OK;
}

int moe_router_logits(dsmoe_ctx* ctx_, const void* router_packed, const void* x, int32_t T, float* logits, void* stream) {
  Ctx* ctx = reinterpret_cast<Ctx*>(ctx_);
  if (!ctx || T < 0 || !router_packed || ((uintptr_t)router_packed & 15) != 0) return DSMOE_EINVAL;
  if (T > 0 && (!x || !logits || ((uintptr_t)x & 15) != 0)) return DSMOE_EINVAL;
  if (T > ctx->L.max_tokens) return DSMOE_EINVAL;
  hipError_t err = launch_router(ctx->L, T, (const char*)router_packed, x, logits, (hipStream_t)stream);
  if (err != hipSuccess) return hip_fail(ctx, err);
  return DSMOE_OK;
}

int moe_dualsparse_forward_routed(dsmoe_ctx* ctx_, const void* packed, const void* router_packed, const void* x,
                                  const float* tau, int32_t T, void* y, float* logits_out, void* workspace, void* stream) {
  Ctx* ctx = reinterpret_cast<Ctx*>(ctx_);
  if (!ctx || T < 0 || !packed || !router_packed || !tau || !workspace) return DSMOE_EINVAL;
  if (T > 0 && (!x || !y || ((uintptr_t)x & 15) != 0)) return DSMOE_EINVAL;
  if (((uintptr_t)workspace & 255) != 0 || ((uintptr_t)packed & 15) != 0 || ((uintptr_t)router_packed & 15) != 0) return DSMOE_EINVAL;
  if (T > ctx->L.max_tokens) return DSMOE_EINVAL;
  float* lbuf = logits_out ? logits_out : (float*)((char*)workspace + ctx->L.o_logits);
  return forward_impl(ctx, ctx->L, packed, (const char*)router_packed, x, lbuf, tau, T, y, workspace, stream);
}

int moe_transform_complete(dsmoe_ctx* ctx_, const void* wg, const void* w1, const void* w3, const void* w2,
                           const int32_t* perm, void* wg_out, void* w1_out, void* w3_out, void* w2_out, void* workspace,
                           void* stream) {
  Ctx* ctx = reinterpret_cast<Ctx*>(ctx_);
  if (!ctx || !w1 || !w3 || !w2 || !w1_out || !w3_out || !w2_out) return DSMOE_EINVAL;
  if ((wg == nullptr) != (wg_out == nullptr)) return DSMOE_EINVAL;
  if (perm && (!workspace || ((uintptr_t)workspace & 255) != 0)) return DSMOE_EINVAL;
  const Layout& L = ctx->L;
  hipStream_t s = (hipStream_t)stream;
  hipError_t err;
  if (perm) {
    int32_t* scratch = (int32_t*)((char*)workspace + L.o_perm_check);
    err = launch_perm_check(L, perm, scratch, s);
    if (err != hipSuccess) return hip_fail(ctx, err);
    int32_t bad = 0;
    err = hipMemcpyAsync(&bad, scratch + (size_t)L.E_res * L.F, sizeof(int32_t), hipMemcpyDeviceToHost, s);
    if (err != hipSuccess) return hip_fail(ctx, err);
    err = hipStreamSynchronize(s);
    if (err != hipSuccess) return hip_fail(ctx, err);
    if (bad != 0) return DSMOE_EPERM;
  }
  err = launch_transform_complete(L, wg, w1, w3, w2, perm, wg_out, w1_out, w3_out, w2_out, s);
  if (err != hipSuccess) return hip_fail(ctx, err);
  return DSMOE_OK;
}

int dsmoe_profile_begin(dsmoe_ctx* ctx_, int level, int max_calls) {
  Ctx* ctx = reinterpret_cast<Ctx*>(ctx_);
  if (!ctx || level < 1 || level > 2 || max_calls < 1 || max_calls > 100000) return DSMOE_EINVAL;
  Profile& pf = ctx->prof;
  if (pf.ev) return DSMOE_EINVAL;  // already profiling
  const int per_call = level == 2 ? kNumKernels + 1 : 2;
  const size_t n = (size_t)per_call * max_calls;
  pf.ev = (hipEvent_t*)calloc(n, sizeof(hipEvent_t));
  if (!pf.ev) return DSMOE_EINVAL;
  for (size_t i = 0; i < n; ++i) {
    hipError_t e = hipEventCreate(&pf.ev[i]);
    if (e != hipSuccess) {
      for (size_t j = 0; j < i; ++j) (void)hipEventDestroy(pf.ev[j]);
      free(pf.ev);
      pf.ev = nullptr;
      return hip_fail(ctx, e);
    }
  }
  pf.level = level;
  pf.max_calls = max_calls;
  pf.calls = 0;
  return DSMOE_OK;
}

int dsmoe_profile_end(dsmoe_ctx* ctx_, float* ms, int* calls) {
  Ctx* ctx = reinterpret_cast<Ctx*>(ctx_);
  if (!ctx || !ms || !calls) return DSMOE_EINVAL;
  Profile& pf = ctx->prof;
  if (!pf.ev) return DSMOE_EINVAL;
  const int per_call = pf.level == 2 ? kNumKernels + 1 : 2;
  double sum[kNumKernels] = {0};
  int rc = DSMOE_OK;
  for (int c = 0; c < pf.calls && rc == DSMOE_OK; ++c) {
    hipEvent_t* ev = pf.ev + (size_t)c * per_call;
    hipError_t e = hipEventSynchronize(ev[per_call - 1]);
    if (e != hipSuccess) {
      rc = hip_fail(ctx, e);
      break;
    }
    if (pf.level == 2) {
      for (int k = 0; k < kNumKernels; ++k) {
        float t = 0.f;
        e = hipEventElapsedTime(&t, ev[k], ev[k + 1]);
        if (e != hipSuccess) {
          rc = hip_fail(ctx, e);
          break;
        }
        sum[k] += t;
      }
    } else {
      float t = 0.f;
      e = hipEventElapsedTime(&t, ev[0], ev[1]);
      if (e != hipSuccess) rc = hip_fail(ctx, e);
      sum[4] += t;
    }
  }
  for (int k = 0; k < kNumKernels; ++k) ms[k] = pf.calls > 0 ? (float)(sum[k] / pf.calls) : 0.f;
  *calls = pf.calls;
  const size_t n = (size_t)per_call * pf.max_calls;
  for (size_t i = 0; i < n; ++i) (void)hipEventDestroy(pf.ev[i]);
  free(pf.ev);
  pf = Profile();
  return rc;
}

int moe_profile_importance(dsmoe_ctx* ctx_, const void* packed, const void* x, const float* logits, int32_t T, int32_t metric,
                           float* importance, void* workspace, void* stream) {
  Ctx* ctx = reinterpret_cast<Ctx*>(ctx_);
  if (!ctx || T < 0 || !packed || !importance || !workspace || metric < 0 || metric > 3) return DSMOE_EINVAL;
  if (T > 0 && (!x || !logits)) return DSMOE_EINVAL;
  if (((uintptr_t)workspace & 255) != 0) return DSMOE_EINVAL;
  if (T > ctx->L.max_tokens) return DSMOE_EINVAL;
  Layout L = ctx->L;  // per-call boundary of the shared rows, as in the forward call
  L.tall_tiles = 0;   // the profiling variant of GEMM-1 has no tall form
  L.sh_rows = L.n_shared > 0 ? (int)align_up(T, L.BM) : 0;
  ctx->last_sh_rows = L.sh_rows;
  hipStream_t s = (hipStream_t)stream;
  char* ws = (char*)workspace;
  // every routed pair takes part: thresholds of zero keep all units
  hipError_t err = launch_fill_i32((int32_t*)(ws + L.o_tau0), (int64_t)L.E * L.P, 0, s);
  if (err == hipSuccess && T > 0)
    err = launch_route(L, logits, T, (const float*)(ws + L.o_tau0), (int32_t*)(ws + L.o_idx), (float*)(ws + L.o_w),
                       (uint8_t*)(ws + L.o_keep), (int32_t*)(ws + L.o_bin_count), nullptr, s);
  if (err == hipSuccess) err = launch_plan(L, T, ws, s);
  if (err == hipSuccess) err = launch_scatter(L, T, ws, s);
  if (err == hipSuccess)
    err = L.mfma ? launch_gemm1_mfma(L, T, (const char*)packed, x, ws, 1 + metric, s)
                 : launch_gemm1_generic(L, T, (const char*)packed, x, ws, 1 + metric, s);
  if (err == hipSuccess) err = launch_colsum(L, ws, metric, importance, s);
  if (err != hipSuccess) return hip_fail(ctx, err);
  return DSMOE_OK;
}

int moe_importance_to_perm(dsmoe_ctx* ctx_, const float* importance, int32_t* perm, void* stream) {
  Ctx* ctx = reinterpret_cast<Ctx*>(ctx_);
  if (!ctx || !importance || !perm) return DSMOE_EINVAL;
  hipError_t err = launch_perm_from_importance(ctx->L, importance, perm, (hipStream_t)stream);
  if (err != hipSuccess) return hip_fail(ctx, err);
  return DSMOE_OK;
}

int moe_select_thresholds(dsmoe_ctx* ctx_, const float* logits, int32_t T, const float* tau_max, int32_t group_size,
                          int32_t row_cap, float* tau, int32_t* pair_count, void* workspace, void* stream) {
  Ctx* ctx = reinterpret_cast<Ctx*>(ctx_);
  if (!ctx || T < 0 || !tau_max || !tau || !workspace || row_cap < 0) return DSMOE_EINVAL;
  if (T > 0 && !logits) return DSMOE_EINVAL;
  if (((uintptr_t)workspace & 255) != 0) return DSMOE_EINVAL;
  const Layout& L = ctx->L;
  if (T > L.max_tokens || group_size < 1 || L.E % group_size != 0) return DSMOE_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  char* ws = (char*)workspace;
  // zero thresholds for the routing pass and a cleared score histogram (adjacent in the workspace)
  const int64_t clear = (L.o_sel - L.o_tau0) / 4 + (int64_t)(L.E + 1) * (kSelBins + 2);
  hipError_t err = launch_fill_i32((int32_t*)(ws + L.o_tau0), clear, 0, s);
  if (err == hipSuccess && T > 0)
    err = launch_route(L, logits, T, (const float*)(ws + L.o_tau0), (int32_t*)(ws + L.o_idx), (float*)(ws + L.o_w),
                       (uint8_t*)(ws + L.o_keep), nullptr, nullptr, s, true);
  if (err == hipSuccess) err = launch_select_thresholds(L, T, tau_max, group_size, row_cap, ws, tau, pair_count, s);
  if (err != hipSuccess) return hip_fail(ctx, err);
  return DSMOE_OK;
}

int moe_thresholds_for_drop_rate(dsmoe_ctx* ctx_, const float* logits, int32_t T, double rate, const int32_t* offset_bins,
                                 float* tau, int32_t* stats, void* workspace, void* stream) {
  Ctx* ctx = reinterpret_cast<Ctx*>(ctx_);
  if (!ctx || T < 0 || !offset_bins || !tau || !workspace || !(rate >= 0.0 && rate <= 1.0)) return DSMOE_EINVAL;
  if (T > 0 && !logits) return DSMOE_EINVAL;
  if (((uintptr_t)workspace & 255) != 0) return DSMOE_EINVAL;
  const Layout& L = ctx->L;
  if (T > L.max_tokens) return DSMOE_EINVAL;
  for (int p = 0; p < L.P; ++p)
    if (offset_bins[p] < -kSelBins || offset_bins[p] > kSelBins) return DSMOE_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  char* ws = (char*)workspace;
  // zero thresholds for the routing pass; of the score histograms only the resident row is used here
  hipError_t err = launch_fill_i32((int32_t*)(ws + L.o_tau0), (int64_t)L.E * L.P, 0, s);
  if (err == hipSuccess)
    err = launch_fill_i32((int32_t*)(ws + L.o_sel) + (int64_t)L.E * (kSelBins + 2), kSelBins + 2, 0, s);
  if (err == hipSuccess && T > 0)
    err = launch_route(L, logits, T, (const float*)(ws + L.o_tau0), (int32_t*)(ws + L.o_idx), (float*)(ws + L.o_w),
                       (uint8_t*)(ws + L.o_keep), nullptr, nullptr, s, true);
  if (err == hipSuccess) err = launch_drop_rate_thresholds(L, T, rate, offset_bins, ws, tau, stats, s);
  if (err != hipSuccess) return hip_fail(ctx, err);
  return DSMOE_OK;
}

int dsmoe_plan_layout(const dsmoe_ctx* ctx_, int64_t* out) {
  const Ctx* ctx = reinterpret_cast<const Ctx*>(ctx_);
  if (!ctx || !out) return DSMOE_EINVAL;
  const Layout& L = ctx->L;
  out[0] = L.o_idx;
  out[1] = L.o_w;
  out[2] = L.o_keep;
  out[3] = L.o_pair_row;
  out[4] = L.o_row_token;
  out[5] = L.o_row_bits;
  out[6] = L.o_exp_nrows;
  out[7] = L.o_exp_row0;
  out[8] = L.row_cap;
  out[9] = L.BM;
  out[10] = ctx->last_sh_rows;
  out[11] = L.o_counters;
  out[12] = L.o_items1;
  out[13] = L.o_items2;
  return DSMOE_PLAN_FIELDS;
}

}  // extern "C"
