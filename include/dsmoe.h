/*
 * dsmoe.h - C ABI of libdsmoe: forward pass of a partitioned, computation-dropping MoE FFN layer
 * on one AMD MI355X (gfx950).
 *
 * The layer (DualSparse-MoE, arXiv 2508.18376):
 *   gating      s = Softmax(router logits), Top-K experts per token            (Sec. 2.1.1, Eq. 1-2)
 *   experts     f_e(x) = (Swish(x W1_e) * (x W3_e)) W2_e                       (Sec. 2.1.1, Eq. 4)
 *   partition   expert e's neurons, put in the order of a static permutation (most important
 *               first), are split evenly into P contiguous sub-experts e*P .. e*P+P-1; every
 *               sub-expert inherits the gate score of its expert, W2 is not rescaled
 *                                                                    (Sec. 3.2; Sec. 4.2 a, b)
 *   dropping    n = score normalised over the K selected experts; unit (token, expert e,
 *               partition p) is computed iff n >= tau[e][p]; tau equal across p is the single-
 *               threshold drop, tau[.][0] < tau[.][1] the dual-threshold drop; per-expert rows of
 *               tau carry load-aware thresholds                    (Sec. 4.1; Sec. 4.2 c; Sec. 4.3)
 *   output      y = sum over kept units of g_e * f_{e,p}(x) (+ always-on shared experts), with
 *               g_e the ORIGINAL gate score (or n, for models that normalise)   (Eq. 3; Sec. 4.1)
 *
 * Conventions
 *   - Every pointer named "device" below is GPU memory on the current HIP device, owned by the
 *     caller; the library allocates no device memory and keeps no reference after the call's
 *     kernels have run.  "stream" is a hipStream_t passed as void* (NULL = the default stream).
 *   - All calls return 0 (DSMOE_OK) or a negative dsmoe_status; they never throw.
 *   - moe_route_and_mask and moe_dualsparse_forward only enqueue kernels: no host
 *     synchronisation, no allocation.  moe_partition_weights synchronises the stream once
 *     (it reads back the permutation check).
 *   - NaN router logits give unspecified routing (not an error): a NaN logit ranks last, every token
 *     still gets K distinct expert ids in range, and no later step leaves its buffers.
 *   - A context keeps a little host-side state per call (profiling events, the last plan's row
 *     layout): host threads must not call into the SAME context at the same time.  Several
 *     contexts, each with its own workspace, may run concurrently on different streams.
 *   - The library reads no environment variable; which kernels a context runs follows from its
 *     dsmoe_config alone (see dsmoe_uses_mfma).
 */
#ifndef DSMOE_H
#define DSMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dsmoe_ctx dsmoe_ctx; /* opaque; host memory owned by the library */

typedef enum { DSMOE_F32 = 0, DSMOE_BF16 = 1 } dsmoe_dtype;

typedef enum {
  DSMOE_OK = 0,
  DSMOE_EINVAL = -1, /* bad shape, divisibility, limit, NULL pointer, T > max_tokens */
  DSMOE_EPERM = -2,  /* perm is not a permutation of 0..d_ff-1 for some expert */
  DSMOE_ENOSPC = -3, /* moe_dualsparse_forward_static: the batch does not fit the static scratch array */
  DSMOE_EHIP = -4    /* a HIP call or kernel launch failed; see dsmoe_last_hip_error */
} dsmoe_status;

typedef struct {
  int32_t d_model;        /* D */
  int32_t d_ff;           /* F: neurons of one routed expert; F % n_part == 0 */
  int32_t n_experts;      /* E: width of the router (all experts of the layer), 1..512 */
  int32_t top_k;          /* K: 1..min(E,16) */
  int32_t n_part;         /* P: sub-experts per expert, 1..8 */
  int32_t n_shared;       /* always-on experts (0 if none) */
  int32_t d_ff_shared;    /* neurons of one shared expert */
  int32_t expert_lo;      /* routed experts [expert_lo, expert_hi) are resident on this GPU; */
  int32_t expert_hi;      /*   pairs routed elsewhere contribute nothing here. [0,E) = all */
  int32_t renorm_combine; /* 0: combine weight = softmax score (Eq. 2); 1: = normalised score */
  int32_t max_tokens;     /* largest T of any later call; sizes the workspace */
  int32_t dtype;          /* dsmoe_dtype of x, weights and y */
  int32_t y_fp32;         /* 1: y is float [T][D] although dtype is DSMOE_BF16 (the fp32 sum of Eq. 3 is stored
                             unrounded); 0: y has the layer's dtype.  No effect on DSMOE_F32 layers. */
  int32_t h_scale_log2;   /* k in [-40, 40], normally 0.  On the matrix-core path the intermediate activation
                             h = Swish(x W1) * (x W3) is held in half precision as h * 2^k: full precision for
                             6.1e-5 <= |h| * 2^k <= 65504, saturation above, an absolute error of 3e-8 below.
                             Layers whose activations are far from 1 in magnitude choose k to centre them.  The
                             factor is folded into the packed weights and taken out again exactly: it changes
                             nothing else and costs nothing per call. */
  int32_t partial_fp32;   /* 0 (normal): on the matrix-core path the per-(token, expert) partial outputs that the
                             combine step adds up are stored in half precision (11 significant bits each), scaled
                             relative to the largest |W2| and to h * 2^k of h_scale_log2: full precision over some
                             seven decades below their typical size, saturation a factor 60 and more above it.
                             They are the largest memory stream of layers with many experts per token.
                             1: they are kept in fp32.  Sums are fp32 either way. */
  int32_t tall_items;     /* Matrix-core path only; the results are the same either way.  An expert's last tile of at
                             most 64 rows can be computed by the work items of the full tile before it ("tall" items)
                             instead of by items of its own.  0 (normal): the plan decides per batch, from the number
                             and length of the items either list would have; 1: wherever it is possible; -1: never. */
} dsmoe_config;

/* Validates cfg and builds the host-side context.  No GPU call is made. */
int dsmoe_create(const dsmoe_config* cfg, dsmoe_ctx** out);
int dsmoe_destroy(dsmoe_ctx* ctx);

/* Bytes of the packed-weight buffer / of the workspace the caller must allocate (device). */
size_t dsmoe_packed_bytes(const dsmoe_ctx* ctx);
size_t dsmoe_workspace_bytes(const dsmoe_ctx* ctx);

const char* dsmoe_strerror(int status);
/* hipError_t value of the last failed HIP call on this context (0 if none). */
int dsmoe_last_hip_error(const dsmoe_ctx* ctx);
/* 1 if this context runs the bf16 MFMA kernels, 0 if it runs the generic fp32-accumulate kernels
 * (fp32 layers, bf16 layers whose D, F/P or shared width is not a multiple of 32, or contexts whose
 * max_tokens * D * 2 bytes of activations reach 2 GiB: split such batches). */
int dsmoe_uses_mfma(const dsmoe_ctx* ctx);

/*
 * Expert partition + reconstruction, once per layer (Sec. 3.2: even split into P sub-experts,
 * no W2 scaling; Sec. 4.2 b: neurons reorganised by a static importance order).
 *   w1, w3   device [E_res][D][F]   gate / up projections of the resident experts, row-major
 *   w2       device [E_res][F][D]   down projection           (E_res = expert_hi - expert_lo)
 *   sh_w1, sh_w3 device [n_shared][D][F_sh], sh_w2 device [n_shared][F_sh][D]; NULL iff n_shared == 0
 *   perm     device int32 [E_res][F]: perm[e][j] = ORIGINAL neuron placed at new position j;
 *            sub-expert p owns positions [p*F/P, (p+1)*F/P).  NULL = identity.
 *   packed_out device, dsmoe_packed_bytes(ctx) bytes: receives the weights in the library's
 *            kernel layout; inputs are not modified.
 * Returns DSMOE_EPERM (packed_out contents then undefined) if perm is not a permutation.
 */
int moe_partition_weights(dsmoe_ctx* ctx, const void* w1, const void* w3, const void* w2, const void* sh_w1,
                          const void* sh_w3, const void* sh_w2, const int32_t* perm, void* packed_out, void* stream);

/*
 * Gating, Top-K and drop mask (Eq. 1-2; Sec. 4.1; Sec. 4.2 c; index remap of Sec. 3.2).
 *   logits  device float [T][E]
 *   tau     device float [E][P], row = global expert id, column = partition (0 = major)
 *   topk_idx   device int32 [T][K]  expert ids by (logit descending, index ascending)
 *   topk_w     device float [T][K]  combine weight g (see renorm_combine)
 *   keep_bits  device uint8 [T][K]  bit p set iff unit (t, k, p) is kept; 0 for non-resident experts
 *   group_count device int32 [E*P]  kept units of sub-expert e*P+p
 * T may be 0.  Arithmetic is fp32; the keep decision is (n >= tau) in fp32.
 */
int moe_route_and_mask(dsmoe_ctx* ctx, const float* logits, int32_t T, const float* tau, int32_t* topk_idx,
                       float* topk_w, uint8_t* keep_bits, int32_t* group_count, void* stream);

/*
 * The whole layer: gating + mask, compacted per-expert row lists, grouped GEMM gate/up with
 * Swish*mul, grouped GEMM down over the kept partitions only, gate-weighted combine (Eq. 1-4 with
 * the dropped units of Sec. 4 removed).
 *   packed  device, written by moe_partition_weights for this ctx
 *   x       device [T][D] (cfg.dtype), logits device float [T][E], tau device float [E][P]
 *   y       device [T][D] (cfg.dtype, or float if cfg.y_fp32), fully overwritten; a token with every
 *           unit dropped gets exact zeros (plus the shared experts' output)
 *   workspace device, >= dsmoe_workspace_bytes(ctx), 256-byte aligned; contents need not be
 *           preserved between calls; two calls that overlap in time need two workspaces
 * bf16 layers accumulate in fp32 and round the output once.  On the matrix-core path the
 * intermediate activation Swish(x W1) * (x W3) is stored in IEEE half precision (values beyond
 * +-65504 saturate) and multiplied with W2 held as half precision times a per-layer power of two,
 * which represents every bf16 weight within 2^-29 of the largest exactly, and the per-pair partial
 * outputs are stored in half precision unless cfg.partial_fp32 is set; bf16 layers on the generic path
 * (see dsmoe_uses_mfma) keep both in fp32.
 */
int moe_dualsparse_forward(dsmoe_ctx* ctx, const void* packed, const void* x, const float* logits, const float* tau,
                           int32_t T, void* y, void* workspace, void* stream);

/*
 * moe_dualsparse_forward for callers that cannot allocate or hand over device memory for a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, same kernels and same results as moe_dualsparse_forward, minus the workspace: the
 * kernels use a static array of DSMOE_STATIC_SCRATCH_BYTES of device memory that is part of the
 * loaded library (every GPU the library runs on holds its own copy until the process ends).  The
 * call allocates and frees nothing and does not synchronise.
 *   - The workspace is laid out for this call's T (not for cfg.max_tokens); a batch that needs more
 *     than the array returns DSMOE_ENOSPC and launches nothing.  dsmoe_static_workspace_need(ctx, T)
 *     tells the bytes a batch of T tokens takes (0 for an invalid argument).  Decode-sized batches of
 *     the large layers fit (a Mixtral-shaped layer up to about 900 tokens).
 *   - The first call on a device looks the array's address up (no allocation, but a runtime query):
 *     make one call with T = 0 before a graph capture starts.
 *   - Every call on a GPU uses that GPU's one array and overwrites what the last call left: calls
 *     that overlap in time on one GPU (two streams, two host threads, two contexts) race.  Run them
 *     one after the other, or give the overlapping ones moe_dualsparse_forward with own workspaces.
 *   - dsmoe_plan_layout describes the caller's workspace, not this array.
 */
#define DSMOE_STATIC_SCRATCH_BYTES (256u << 20)
int moe_dualsparse_forward_static(dsmoe_ctx* ctx, const void* packed, const void* x, const float* logits, const float* tau,
                                  int32_t T, void* y, void* stream);
size_t dsmoe_static_workspace_need(const dsmoe_ctx* ctx, int32_t T);

/*
 * Gating logits l = x W_g (Sec. 3.1, first equation; the input of Eq. 1).
 *   moe_pack_router: wg device [D][E] (cfg.dtype), row-major as in the paper; router_packed device,
 *     dsmoe_router_packed_bytes(ctx) bytes, 16-byte aligned: W_g in the kernel's operand order
 *     (once per layer).  Asynchronous.
 *   moe_router_logits: x device [T][D] (cfg.dtype, 16-byte aligned); logits device float [T][E],
 *     fully overwritten.  Products are exact, accumulation is fp32 (order differs from a sequential
 *     sum).  Asynchronous, no allocation.
 *   moe_dualsparse_forward_routed: moe_router_logits followed by moe_dualsparse_forward on those
 *     logits; logits_out device float [T][E] receives them, or NULL to keep them in the workspace.
 */
size_t dsmoe_router_packed_bytes(const dsmoe_ctx* ctx);
int moe_pack_router(dsmoe_ctx* ctx, const void* wg, void* router_packed, void* stream);
int moe_router_logits(dsmoe_ctx* ctx, const void* router_packed, const void* x, int32_t T, float* logits, void* stream);
int moe_dualsparse_forward_routed(dsmoe_ctx* ctx, const void* packed, const void* router_packed, const void* x,
                                  const float* tau, int32_t T, void* y, float* logits_out, void* workspace, void* stream);

/*
 * Complete transformation (Sec. 3.1, steps 1-3): rewrites the layer described by ctx (E experts of
 * F neurons, P parts) as a plain layer of E*P experts of F/P neurons that any MoE implementation,
 * this library included (n_experts = E*P, top_k = K*P, n_part = 1), runs with Top-(K*P) and that
 * computes the same output.
 *   wg   device [D][E] or NULL (then wg_out must be NULL too)   -> wg_out device [D][E*P]: column e
 *        repeated P times (new experts e*P .. e*P+P-1)
 *   w1, w3 device [E_res][D][F] -> w1_out, w3_out device [E_res*P][D][F/P]
 *   w2   device [E_res][F][D]   -> w2_out device [E_res*P][F/P][D], multiplied by P (one rounding to
 *        cfg.dtype; exact for P = 2, 4, 8)
 *   perm device int32 [E_res][F] or NULL, as for moe_partition_weights: new expert e*P+p gets the
 *        original neurons perm[e][p*F/P .. (p+1)*F/P - 1] in that order (Sec. 4.2 b)
 *   workspace: needed only with perm (the permutation check); as for moe_dualsparse_forward.
 * Outputs must not overlap inputs.  With perm the call synchronises the stream once and returns
 * DSMOE_EPERM for a non-permutation (outputs then untouched); otherwise asynchronous.
 */
int moe_transform_complete(dsmoe_ctx* ctx, const void* wg, const void* w1, const void* w3, const void* w2,
                           const int32_t* perm, void* wg_out, void* w1_out, void* w3_out, void* w2_out, void* workspace,
                           void* stream);

/*
 * Neuron importance profiling on calibration tokens (Sec. 4.2 b): for every resident expert e and
 * ORIGINAL neuron q, the sum over the calibration tokens routed to e (Top-K, nothing dropped) of
 *   metric 0  Swish(x W1_q)            1  |Swish(x W1_q)|
 *   metric 2  Swish(x W1_q) (x W3_q)   3  |Swish(x W1_q) (x W3_q)|
 *   packed      device, made by moe_partition_weights with perm == NULL (identity) for this ctx
 *   x, logits   device [T][D] / float [T][E]: the calibration tokens
 *   importance  device float [E_res][F], fully overwritten (0 for an expert no token routes to)
 *   workspace   as for moe_dualsparse_forward (its contents are overwritten)
 * Terms and sums are fp32.  The rows of a tile are summed in the order the row list holds them, which
 * can differ between runs (see moe_dualsparse_forward's row lists): the last bits of a sum may too.
 * Asynchronous, no allocation.
 */
int moe_profile_importance(dsmoe_ctx* ctx, const void* packed, const void* x, const float* logits, int32_t T,
                           int32_t metric, float* importance, void* workspace, void* stream);

/*
 * Reconstruction order from an importance table (Sec. 4.2 b: the major sub-expert takes the most
 * important neurons): perm[e][j] = neuron with the j-th largest importance[e][.], equal values by
 * ascending neuron id.  importance device float [E_res][F], perm device int32 [E_res][F].  The
 * result is what moe_partition_weights takes as perm.  A NaN importance ranks as minus infinity (last).
 */
int moe_importance_to_perm(dsmoe_ctx* ctx, const float* importance, int32_t* perm, void* stream);

/*
 * Load-aware thresholds chosen on the device, without a host round trip (Sec. 4.3; Sec. 5.3.3 on
 * the non-linear relation between threshold and drop rate).  Routes the batch over the whole
 * router with nothing dropped and writes the table moe_dualsparse_forward takes as tau:
 *   1. device d holds experts [d*group_size, (d+1)*group_size) (group_size divides E); its load
 *      ratio is r = pairs routed to its experts / (T*K*group_size/E); its experts get
 *      tau_max[p] * min(r, 1): the predefined maximum where the load is at or above the balanced
 *      share, proportionally less below it;
 *   2. if row_cap > 0: for every expert whose lowest threshold would let more than row_cap of its
 *      pairs through, all its thresholds are lifted by the same amount so that the lowest becomes
 *      the smallest multiple of 2^-12 that at most row_cap of its pairs reach (above 1, i.e. drop
 *      everything, if more than row_cap pairs have score 1).
 *   logits device float [T][E]; tau_max device float [P]; tau device float [E][P] (output);
 *   pair_count device int32 [E] (output, may be NULL): Top-K pairs per expert before any drop;
 *   workspace as for moe_dualsparse_forward (overwritten).  Arithmetic is fp32 with one rounding
 *   per operation.  T == 0 gives tau_max everywhere.  Asynchronous, no allocation.
 */
int moe_select_thresholds(dsmoe_ctx* ctx, const float* logits, int32_t T, const float* tau_max, int32_t group_size,
                          int32_t row_cap, float* tau, int32_t* pair_count, void* workspace, void* stream);

/*
 * Thresholds for a target drop rate, chosen on the device from the batch's own score distribution
 * (Sec. 5.3.3: the relation between threshold and drop rate is not linear; Sec. 4.2 c: the
 * partitions' thresholds keep fixed offsets around a centre, e.g. T - 0.01 / T + 0.01).
 *   Thresholds live on the grid of multiples of 2^-12: tau[e][p] = (b + offset_bins[p]) / 4096, the
 *   same row for every expert.  b is the smallest integer for which at least rate * (resident pairs
 *   * P) units of the pairs routed to the resident experts fall below their threshold.
 *   logits device float [T][E]; rate in [0, 1] (the count rate * units is formed in double precision);
 *   offset_bins HOST int32 [P], each in [-4096, 4096]
 *   (0.01 is 41 grid steps); tau device float [E][P] (output);
 *   stats device int32 [2] (output, may be NULL): dropped units, resident pairs * P.
 *   workspace as for moe_dualsparse_forward (overwritten).  Asynchronous, no allocation.
 */
int moe_thresholds_for_drop_rate(dsmoe_ctx* ctx, const float* logits, int32_t T, double rate, const int32_t* offset_bins,
                                 float* tau, int32_t* stats, void* workspace, void* stream);

/*
 * Inspection of the last forward call's plan, for tests: byte offsets into the workspace.
 * Fills out[0..DSMOE_PLAN_FIELDS-1]; returns the number of fields.
 *   0 topk_idx int32[T*K]      1 topk_w float[T*K]        2 keep_bits uint8[T*K]
 *   3 pair_row int32[T*K] (-1 = no kept unit)              4 row_token int32[rows]
 *   5 row_bits uint8[rows]     6 expert_nrows int32[E_res] 7 expert_row0 int32[E_res]
 *   8 row capacity (a count, not an offset)                9 row tile height (a count)
 *  10 rows at the start of the row space that the last call gave to the shared experts (a count)
 *  11 counters int32[5]: items of GEMM-1, items of GEMM-2, row tiles that have GEMM-2 items, K ranges GEMM-2 is
 *     split into, first row tile (in row order) with a split item
 *  12 work list of the first grouped GEMM, counters[0] records of 8 int32: first row, rows the item multiplies, expert
 *     (resident index; the number of resident experts = the shared experts), partition, neuron tile, rows it writes
 *     (the rest zeros), half (0 whole neuron tile, 1 / 2 its first / second 64 neurons), unused
 *  13 work list of the second grouped GEMM, counters[1] records of 8 int32: first row, rows, expert, output column
 *     tile, bit mask of the partitions it sums over, first K stage and number of K stages inside every such
 *     partition, 0 or 1 + the partial-output tile it writes instead of the rows of the per-pair output
 * (fields 12 and 13 describe the lists of the matrix-core path and of the generic path alike)
 */
#define DSMOE_PLAN_FIELDS 14
int dsmoe_plan_layout(const dsmoe_ctx* ctx, int64_t* out);

/*
 * Per-kernel timing of the next moe_dualsparse_forward calls on this context, for benchmarks.
 * The steps of the layer (Eq. 1-4 with the drops of Sec. 4) run as up to seven kernels: router
 * (only in moe_dualsparse_forward_routed; otherwise its slot reads 0), route+mask, plan, scatter,
 * GEMM-1, GEMM-2, combine.  begin creates HIP events (host objects, no
 * device memory); while profiling, forward records them on its stream between the kernels
 * (level 2) or only around GEMM-1 (level 1) and stays asynchronous; calls beyond max_calls are not
 * recorded.  end waits for the recorded events, writes the mean duration in milliseconds of each
 * kernel to ms[0..6] (host memory; 0 where not recorded) and the number of recorded calls to
 * *calls, destroys the events and switches profiling off.
 */
#define DSMOE_NUM_KERNELS 7
int dsmoe_profile_begin(dsmoe_ctx* ctx, int level, int max_calls);
int dsmoe_profile_end(dsmoe_ctx* ctx, float* ms, int* calls);

#ifdef __cplusplus
}
#endif
#endif /* DSMOE_H */
