/*
 * hbp.h — C ABI of the MI355X (gfx950) packed varlen causal attention library.
 *
 * One packed buffer holds many samples of different lengths back to back; every token attends
 * only inside its own sample (block-diagonal causal mask given by cu_seqlens).  This is where
 * the attention complexity of a pack, sum_i s_i^2, is spent (paper: Section 1, third
 * paragraph; Section 3.1, ABR paragraph; Appendix D, layer cost 24Bsh^2 + 4B*sum s_i^2).
 *
 * Conventions
 *  - Plain C.  Every function returns an hbp_status (0 = HBP_OK) and never throws or aborts.
 *  - The caller owns every buffer.  The library allocates no device memory, never
 *    synchronises the device and uses only the caller's workspace for scratch.
 *  - "host" / "device" on a pointer says where the memory must live.
 *  - Device entry points enqueue work on the caller's HIP stream (a hipStream_t passed as
 *    void*; NULL = the default stream) and return without waiting.
 *  - Layouts ("thd"): Q [T,Hq,d_qk], K [T,Hkv,d_qk], V [T,Hkv,d_v], O/dO [T,Hq,d_v],
 *    dQ like Q, dK like K, dV like V: bf16, innermost dimension contiguous, token and head
 *    strides in elements (0 = dense).  LSE [Hq,T] fp32 dense.  cu_seqlens int32 [n_samples+1].
 *  - Query head h reads kv head h / (Hq/Hkv) (contiguous groups).
 *  - Supported head dims (d_qk, d_v): (64,64), (128,128), (192,128).
 */
#ifndef HBP_H
#define HBP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t hbp_status;
enum {
  HBP_OK = 0,
  HBP_ERR_INVALID_ARG = 1, /* null pointer, non-positive size, bad enum value            */
  HBP_ERR_SHAPE = 2,       /* Hq % Hkv != 0, stride smaller than the row it must hold,
                            * not a multiple of 8, or a token stride above 2^22 elements  */
  HBP_ERR_UNSUPPORTED = 3, /* head dims outside the supported set                        */
  HBP_ERR_CAPACITY = 4,    /* an output array of the planner is too small                */
  HBP_ERR_WORKSPACE = 5,   /* workspace missing, misaligned or smaller than required     */
  HBP_ERR_DEVICE = 6,      /* the HIP runtime refused the launch (hipGetLastError)       */
  HBP_ERR_NO_MEMORY = 7,   /* a host planner could not allocate its working memory       */
  HBP_ERR_STATIC_LIMIT = 8 /* hbp_varlen_attn_bwd_static: the problem needs more scratch
                            * than HBP_STATIC_SCRATCH_BYTES                               */
};

/* Static, never-freed description of a status code. */
const char* hbp_status_string(hbp_status s);

/* One work item of a pack: rows [row_begin,row_end) of the packed buffer, all inside sample
 * `sample`, being tile number `tile` of that sample (row_begin = cu[sample] + tile*tile_rows). */
typedef struct {
  int32_t sample, tile, row_begin, row_end;
} hbp_tile;

enum { HBP_TILES_QUERY = 0, HBP_TILES_KEY = 1 };
enum { HBP_FWD = 0, HBP_BWD = 1, HBP_BWD_DQ = 2, HBP_LOSS = 3 }; /* forward; backward (its dK/dV kernel); backward's dQ kernel; the cross-entropy kernel */

/*
 * hbp_pack_plan — host only, integer only, deterministic.
 *
 * Packing of ONE pack (paper Section 4.2 step 1 "Packing", Algorithm 2; the paper allows any
 * packer): walk `lengths` in order, give each sample min(length, space left) tokens, stop when
 * the pack holds pack_len tokens or the list ends (an under-full pack is legal: no padding
 * sample is invented).  Then the Attention Balance Sort of Algorithm 7 applied one level down:
 * cut every sample into tiles of tile_rows rows, give each tile its exact number of causal
 * (query,key) pairs as cost — kind HBP_TILES_QUERY: pairs whose query is in the tile,
 * HBP_TILES_KEY: pairs whose key is in the tile — and sort by (cost descending, sample
 * ascending, tile ascending).  pack_cost is Algorithm 7's a = sum len(x)^2 of the pack.
 *
 * All pointers are HOST memory.  Size query: pass cu_seqlens = NULL and/or tiles = NULL (with
 * tile_cost = NULL); the counts are still written.  Outputs that are non-NULL must have room:
 * cu_cap >= n_samples+1, tile_cap >= n_tiles, else HBP_ERR_CAPACITY (counts still written).
 * Errors: HBP_ERR_INVALID_ARG for lengths == NULL with n_lengths > 0, n_lengths < 0,
 * pack_len <= 0, tile_rows <= 0, bad kind, any length <= 0, NULL count outputs.
 */
hbp_status hbp_pack_plan(const int32_t* lengths, int32_t n_lengths, int32_t pack_len,
                         int32_t tile_rows, int32_t kind,
                         int32_t* cu_seqlens, int32_t cu_cap, int32_t* n_samples_out,
                         int32_t* n_consumed_out,
                         hbp_tile* tiles, int64_t* tile_cost, int32_t tile_cap,
                         int32_t* n_tiles_out, int64_t* pack_cost_out);

/* Problem description shared by forward and backward. */
typedef struct {
  int32_t total_tokens; /* T = cu_seqlens[n_samples]                                   */
  int32_t n_samples;
  int32_t n_q_heads, n_kv_heads;
  int32_t d_qk, d_v;
  float softmax_scale;  /* <= 0: 1/sqrt(d_qk)                                          */
  int32_t fwd_tile_rows; /* rows per tile of the query-tile list given to the FORWARD: 0 = the
                          * hbp_tile_rows value; hbp_fwd_tile_rows() says which larger size, if
                          * any, the forward kernel of this head layout also takes           */
  /* strides in elements; 0 = dense ([T,H,dim] contiguous).  dQ/dK/dV/dO/O use the o_ and
   * the q_/k_/v_ strides of the tensor they mirror (dO and O share o_*).  Every stride is a
   * multiple of 8 (16-byte vector accesses) and holds its row; a token stride is at most
   * 2^22 = 4194304 elements (the kernels address the rows of a tile in 32 bits):
   * HBP_ERR_SHAPE otherwise.                                                           */
  int64_t q_stride_t, q_stride_h, k_stride_t, k_stride_h;
  int64_t v_stride_t, v_stride_h, o_stride_t, o_stride_h;
} hbp_attn_desc;

/* Rows per tile the kernels of this (d_qk, d_v) pair expect from hbp_pack_plan:
 * which = HBP_FWD: query tiles of the forward; HBP_BWD: key tiles of the backward.
 * Returns HBP_ERR_UNSUPPORTED for other head dims. */
hbp_status hbp_tile_rows(int32_t d_qk, int32_t d_v, int32_t which, int32_t* rows_out);

/* Preferred rows per query tile for the FORWARD of this problem (reads the head counts and dims of
 * desc only).  With an odd number of query heads per kv head (multi-head attention included) the
 * forward kernel shares its K/V stream between the two 128-row halves of a 256-row tile instead of
 * between two heads of a group, so 256 is returned; otherwise the hbp_tile_rows value.  A caller
 * that plans the forward's list with this size stores it in desc->fwd_tile_rows; the backward keeps
 * taking a query-tile list made with hbp_tile_rows(..., HBP_FWD). */
hbp_status hbp_fwd_tile_rows(const hbp_attn_desc* desc, int32_t* rows_out);

/* Bytes of device workspace a call needs (256-byte aligned base required).
 * which = HBP_FWD or HBP_BWD.  Forward: the scheduler's per-die queue counters.  Backward: two
 * sets of counters, the per-row D = rowsum(dO*O) and LSE*log2(e), both [Hq,T] fp32; and, with
 * fewer than 8 kv heads, fp32 partial sums of dK and dV, [parts][T][Hkv][d_qk + d_v]: the query
 * heads of a kv head are then dealt out in `parts` runs (the smallest divisor of Hq/Hkv with
 * Hkv * parts >= 8, else Hq/Hkv) that are separate work items, and a reduce kernel adds the parts
 * up in a fixed order (no atomics either way). */
hbp_status hbp_workspace_bytes(const hbp_attn_desc* desc, int32_t which, size_t* bytes_out);

/* Optional per-workgroup record written by the persistent kernels when `profile` != NULL
 * (device memory, hbp_profile_capacity() records). ticks are the 100 MHz constant clock. */
typedef struct {
  uint32_t hw_id;      /* raw HW_ID register of the workgroup's first wave (CU, SE, ...)  */
  uint32_t xcc_id;     /* raw XCC_ID register (accelerator die)                           */
  uint32_t n_items;    /* work items this workgroup processed                             */
  uint32_t reserved;
  uint64_t first_tick; /* when the workgroup took its first item                          */
  uint64_t last_tick;  /* when it finished its last item                                  */
  uint64_t busy_ticks; /* sum over items of (end - start)                                 */
} hbp_profile_rec;

/* Number of hbp_profile_rec the caller must provide = workgroups launched by the kernel named by
 * which (HBP_FWD, HBP_BWD = the dK/dV kernel, HBP_BWD_DQ = the dQ kernel). */
hbp_status hbp_profile_capacity(const hbp_attn_desc* desc, int32_t which, int32_t* n_records_out);

/*
 * hbp_varlen_attn_fwd — O and per-row LSE of causal attention inside each sample.
 *
 *   S[r,k] = scale * <Q[r,h,:], K[k,kh,:]>  for cu[i] <= k <= r < cu[i+1];  kh = h/(Hq/Hkv)
 *   LSE[h,r] = ln sum_k exp(S[r,k]);  O[r,h,:] = sum_k exp(S[r,k]-LSE[h,r]) V[k,kh,:]
 *
 * (standard scaled-dot-product softmax attention; the paper fixes only that attention is per
 * sample inside a pack — Section 1, third paragraph.)  bf16 MFMA with fp32 accumulation,
 * probabilities rounded to bf16 before the PV product, O stored bf16, LSE fp32.
 *
 * q,k,v,o,lse,cu_seqlens,q_tiles,workspace,profile: DEVICE.  desc: HOST.
 * q_tiles: the HBP_TILES_QUERY list of hbp_pack_plan made with hbp_tile_rows(..., HBP_FWD), or
 * with desc->fwd_tile_rows rows when that is set;
 * items are served longest first by a persistent grid.  Tiles that are malformed (outside
 * their sample, longer than the tile size) are skipped, never dereferenced.
 * Rows of O/LSE not covered by any tile are left untouched.  n_q_tiles == 0 or T == 0: no-op.
 * Errors: INVALID_ARG (null pointers, negative counts, n_q_tiles * n_q_heads above INT32_MAX, a
 * fwd_tile_rows the layout does not take), SHAPE, UNSUPPORTED,
 * WORKSPACE, DEVICE.  Nothing is launched when an error is returned.
 */
hbp_status hbp_varlen_attn_fwd(const hbp_attn_desc* desc, const void* q, const void* k,
                               const void* v, const int32_t* cu_seqlens,
                               const hbp_tile* q_tiles, int32_t n_q_tiles,
                               void* o, float* lse,
                               void* workspace, size_t workspace_bytes,
                               hbp_profile_rec* profile_or_null, void* stream);

/*
 * hbp_varlen_attn_bwd — dQ, dK, dV of L = sum(O * dO) for the attention above.
 *
 *   D[r] = sum_x dO[r,h,x] O[r,h,x];  P = exp(S - LSE);  dP[r,k] = <dO[r,h,:], V[k,kh,:]>
 *   dS = P * (dP - D[r]);  dQ = scale * dS K;  dK = scale * sum_{h in group} dS^T Q;
 *   dV = sum_{h in group} P^T dO
 *
 * Three launches on `stream`: a pre-pass (D), the persistent key-tile kernel (dK/dV accumulated in
 * registers over the query blocks and over the query heads of each kv head; followed by a small
 * reduce kernel when there are fewer than 8 kv heads, see hbp_workspace_bytes) and the persistent
 * query-tile kernel (dQ; it recomputes S and dP).  No atomics: every output element is written
 * once, results are bit-stable.
 * q_tiles: the HBP_TILES_QUERY list made with hbp_tile_rows(..., HBP_FWD) (the forward's list
 * unless that was planned with a larger desc->fwd_tile_rows, which the backward ignores);
 * kv_tiles: the HBP_TILES_KEY list made with hbp_tile_rows(..., HBP_BWD).
 * o and lse are the forward's outputs.  dK/dV rows covered by a key tile and dQ rows covered by a
 * query tile are written; others are left untouched.  profile / profile_dq: optional records of
 * the dK/dV and the dQ kernel.  Same memory placement and error rules as the forward.
 */
hbp_status hbp_varlen_attn_bwd(const hbp_attn_desc* desc, const void* q, const void* k,
                               const void* v, const void* o, const float* lse, const void* d_o,
                               const int32_t* cu_seqlens,
                               const hbp_tile* q_tiles, int32_t n_q_tiles,
                               const hbp_tile* kv_tiles, int32_t n_kv_tiles,
                               void* dq, void* dk, void* dv,
                               void* workspace, size_t workspace_bytes,
                               hbp_profile_rec* profile_or_null, hbp_profile_rec* profile_dq_or_null,
                               void* stream);

/*
 * hbp_varlen_attn_bwd_static — the backward above for callers that cannot allocate device memory and
 * have no workspace to hand over: code under HIP graph capture, tight serving or training loops,
 * harnesses that forbid hipMalloc.  Same arguments minus the workspace, same kernels, same results
 * bit for bit.  The scratch (queue counters, D, LSE*log2e and, with fewer than 8 kv heads, the partial
 * sums of dK and dV) lives in a static device array of HBP_STATIC_SCRATCH_BYTES inside the library: each
 * GPU the library runs on holds that much from the moment the library's code is loaded there until
 * the process ends.  The call allocates and frees nothing; the first call on a device looks up the
 * array's address there (make that first call outside a graph capture).
 * Limit: hbp_workspace_bytes(desc, HBP_BWD) must not exceed HBP_STATIC_SCRATCH_BYTES, else
 * HBP_ERR_STATIC_LIMIT and nothing is launched (64 MiB holds n_q_heads * total_tokens up to 8 Mi rows,
 * e.g. 64 heads x 131072 tokens, with 8 or more kv heads).
 * Every call on a GPU uses that GPU's one array: calls that may overlap in time on one GPU (different
 * streams, different host threads) race on it and must be serialised by the caller; calls that follow
 * each other on one stream are safe.  Nothing in the array has to start at zero and nothing is read
 * before this call has written it (the pre-pass resets the counters and fills D and LSE*log2e; the
 * partial sums are written by the key-tile kernel before the reduce kernel reads them), so what an
 * earlier, larger call left behind is never seen.
 * Errors: as hbp_varlen_attn_bwd without HBP_ERR_WORKSPACE, plus HBP_ERR_STATIC_LIMIT, and
 * HBP_ERR_DEVICE when the array's address cannot be obtained.
 */
#define HBP_STATIC_SCRATCH_BYTES ((size_t)((64u << 20) + 4096u))
hbp_status hbp_varlen_attn_bwd_static(const hbp_attn_desc* desc, const void* q, const void* k,
                                      const void* v, const void* o, const float* lse, const void* d_o,
                                      const int32_t* cu_seqlens,
                                      const hbp_tile* q_tiles, int32_t n_q_tiles,
                                      const hbp_tile* kv_tiles, int32_t n_kv_tiles,
                                      void* dq, void* dk, void* dv,
                                      hbp_profile_rec* profile_or_null, hbp_profile_rec* profile_dq_or_null,
                                      void* stream);

/*
 * hbp_set_kernel_events — measurement hook.  When both events are non-NULL, every later call of
 * the entry point that launches the chosen kernel (which = HBP_FWD, HBP_BWD, HBP_BWD_DQ, HBP_LOSS) records
 * `start` on its stream immediately before, and `stop` immediately after, that persistent kernel
 * (the forward kernel; the dK/dV kernel; the dQ kernel), so a caller can time that one launch with
 * hipEventElapsedTime.  Events are hipEvent_t passed as void*, owned by the caller; pass NULLs to
 * switch the hook off.  Process-wide state, not thread safe.  Returns HBP_ERR_INVALID_ARG for a
 * bad `which` or when exactly one event is NULL.
 */
hbp_status hbp_set_kernel_events(int32_t which, void* start_event, void* stop_event);

/* ---- multi-level Balance Packing planner (host only) ------------------------------------------ */

/* one pack: `n_items` sample indices starting at pack_items[first_item] */
typedef struct {
  int32_t level;      /* packing group i (0-based): the pack is filled to at most group_lens[level] */
  int32_t first_item;
  int32_t n_items;
  int32_t n_tokens;   /* sum of the lengths of its samples */
  int64_t attn_cost;  /* attention complexity a = sum len^2 (paper Section 3.1; Attention Balance Sort) */
} hbp_pack;

/* one mini-batch: `n_packs` packs of one level starting at packs[first_pack] (one pack per device) */
typedef struct {
  int32_t level, first_pack, n_packs, reserved;
} hbp_batch;

/* Section 3.1 metrics of a plan (see hbp_balance_packing for how they are evaluated) */
typedef struct {
  double dbr, pr, abr, cr, ave_t;
} hbp_pack_metrics;

/*
 * hbp_balance_packing — the paper's Balance Packing (Section 4.2, Algorithm 2) over a whole dataset
 * of sample lengths.  Host only, integer, deterministic.
 *
 *   GroupData (appendix):  sample x joins group D_i when len(x) is in (l_{i-1}, l_i], l_0 = 0,
 *                          l_i = group_lens[i] (strictly increasing).
 *   for i = n_levels-1 .. 0:
 *     Packing(D_i, l_i):   first-fit decreasing (the paper allows any packer): samples by length
 *                          descending, ties in input order, each into the first pack (creation
 *                          order) it fits.
 *     GreedyFill (appendix): for every pack, for j = i-1 .. 0, for every x still in D_j in input
 *                          order: if tokens(pack) + len(x) <= l_i the sample moves into the pack.
 *     Balance Batching:    attention complexity a = sum len^2 per pack, packs sorted by a
 *                          descending (ties: creation order), cut into runs of packs_per_batch[i]
 *                          packs; a short last run is kept.
 *   Shuffle of all batches: Fisher-Yates from the end with j = r mod (k+1), r from the splitmix64
 *                          stream of shuffle_seed.
 *
 * Outputs, in final order (batches as shuffled, inside a batch the packs in sorted order):
 * batches[n_batches], packs[n_packs], pack_items[n_samples] (every sample index exactly once).
 * Pass pack_items = packs = batches = NULL for a size query (counts and metrics only); otherwise all
 * three must be non-NULL with item_cap >= n_samples, pack_cap / batch_cap >= the counts
 * (HBP_ERR_CAPACITY if not; the counts are still reported).
 * metrics_or_null: one pack is one device's input of an iteration.  DBR and ABR: the equations'
 * sum(v_max - v_i) / (v_max N) over the packs of a batch (v = tokens, resp. a), averaged over the
 * batches of full size; PR = padding / capacity = sum(l_i - tokens) / sum l_i over all packs;
 * CR = tokens in packs of levels with level_sp[i] > 1 over all tokens (level_sp NULL: 0);
 * Ave-T = tokens per pack.
 * Errors: HBP_ERR_INVALID_ARG for NULL counts, n_levels < 1, group_lens not strictly increasing and
 * positive, packs_per_batch[i] < 1, level_sp[i] < 1, a length <= 0 or > the largest group length.
 * All pointers are host memory owned by the caller.
 */
hbp_status hbp_balance_packing(const int32_t* lengths, int32_t n_samples,
                               const int32_t* group_lens, const int32_t* packs_per_batch,
                               const int32_t* level_sp, int32_t n_levels, uint64_t shuffle_seed,
                               int32_t* pack_items, int32_t item_cap,
                               hbp_pack* packs, int32_t pack_cap, int32_t* n_packs_out,
                               hbp_batch* batches, int32_t batch_cap, int32_t* n_batches_out,
                               hbp_pack_metrics* metrics_or_null);

/* ---- hierarchical groups auto-selection ------------------------------------------------------- */

/*
 * Profiling is the caller's (this library does not train a model): two callbacks and a context.
 *   memory(ctx, l, sp, ckpt): REMAINING device memory, any unit, for packing length l, sequence-parallel
 *                             degree sp and ckpt checkpointed layers; negative = does not fit.
 *   time(ctx, l, sp, ckpt):   iteration time; NaN, +inf or negative = cannot run.
 */
typedef struct {
  double (*memory)(void* ctx, int32_t l, int32_t sp, int32_t ckpt);
  double (*time)(void* ctx, int32_t l, int32_t sp, int32_t ckpt);
  void* ctx;
} hbp_profile;

/* Stage 1 result for one candidate length: feasible = 0 when no SP degree fits */
typedef struct {
  int32_t l, sp, ckpt, feasible;
  double time;
} hbp_strategy;

/* one packing group of the result */
typedef struct {
  int32_t l, sp, ckpt, reserved;
} hbp_group;

/*
 * hbp_auto_select — the paper's Hierarchical Groups Auto-Selection (Section 4.1, Algorithm 1) with
 * FindBestSpCkpt and GreedyProfileCkpt of the appendix "Implementation Details of Hierarchical Groups
 * Auto-Selection".  Host only.
 *   GreedyProfileCkpt(l, sp): m1 = memory(l, sp, c_min), m2 = memory(l, sp, c_max),
 *       m_ave = (m2 - m1) / (c_max - c_min), c_o = c_max - m2 / m_ave, taken as a layer count:
 *       ceil, not below 0; m2 < 0: (l, sp) does not fit; m_ave <= 0: 0 if m2 - m_ave c_max >= 0.
 *   FindBestSpCkpt(l): over sp_set in order, time(l, sp, c_o); the first minimum wins.
 *   Stage 1: per_length[i] = FindBestSpCkpt(lengths[i]); j = first argmin of the times;
 *       (s_best, l_best) = entry j, (s_max, l_max) = the last entry (it must be feasible).
 *   Stage 2: l_1 = floor(l_best / s_best.sp), l_2 = floor(l_max / s_max.sp);
 *       groups = {l_1, l_best, l_2, l_max} if l_2 > l_best else {l_1, l_best, l_max}, ascending, a
 *       repeated length reported once.  l_1 and l_2 train with SP 1 and the checkpoint layers of the
 *       strategy they were derived from; l_best and l_max with their own strategy.
 * lengths[n_lengths] strictly increasing and positive, sp_set[n_sp] positive, 0 <= c_min < c_max.
 * Outputs (caller-owned host memory): per_length_or_null[n_lengths], groups[4], *n_groups_out,
 * *best_index_out_or_null = j.
 * Errors: HBP_ERR_INVALID_ARG (NULL pointers or callbacks, bad sets or layer counts),
 * HBP_ERR_UNSUPPORTED when the longest length has no feasible strategy.
 */
hbp_status hbp_auto_select(const int32_t* lengths, int32_t n_lengths, const int32_t* sp_set, int32_t n_sp,
                           int32_t c_min, int32_t c_max, const hbp_profile* profile,
                           hbp_strategy* per_length_or_null, hbp_group* groups, int32_t* n_groups_out,
                           int32_t* best_index_out_or_null);

/* ---- packed cross-entropy with the paper's loss normalisers ------------------------------------ */

enum { HBP_LOSS_TOKEN_MEAN = 0, HBP_LOSS_SAMPLE_MEAN = 1, HBP_LOSS_STABLE = 2 };

/* bytes of device workspace hbp_packed_ce needs (256-byte aligned base) */
hbp_status hbp_packed_ce_workspace_bytes(int32_t total_tokens, int32_t n_samples, size_t* bytes_out);

/*
 * hbp_packed_ce — token cross-entropy over a packed buffer, reduced with one of the normalisers of
 * the paper's Section 4.3 (normaliser equation), and its gradient, in one pass over the logits.
 *
 *   CE_r      = logsumexp(logits[r,:]) - logits[r, labels[r]]          for labels[r] >= 0
 *   loss      = sum_r w_r CE_r
 *   dlogits   = w_r (softmax(logits[r,:]) - onehot(labels[r]))         (zero rows where labels[r] < 0)
 *   w_r       = 1 / sum_i T_i                (HBP_LOSS_TOKEN_MEAN;  T_i = loss tokens of sample i)
 *               1 / (T_i n_samples)          (HBP_LOSS_SAMPLE_MEAN; i = the row's sample)
 *               1 / (n_samples t_ave)        (HBP_LOSS_STABLE; t_ave = the GLOBAL mean of T_i, which the
 *                                             caller reduces over its data-parallel ranks)
 * A batch element of the paper's equation is one sample of the pack (rows cu_seqlens[i] ..
 * cu_seqlens[i+1]), B_l = n_samples.  A sample without loss tokens contributes nothing.
 *
 * All pointers are DEVICE memory owned by the caller: logits bf16 [T, V] with row stride
 * `logit_stride_t` elements (0 = V); labels int32 [T] (negative or >= V: no loss on that token);
 * cu_seqlens int32 [n_samples + 1] with cu_seqlens[0] = 0, cu_seqlens[n_samples] = T;
 * dlogits_or_null bf16 [T, V] dense; loss_out one float; token_loss_or_null float [T] (CE_r, 0 where
 * no label).  V and the stride must be multiples of 8 and the logits 16-byte aligned
 * (HBP_ERR_UNSUPPORTED otherwise).  Rows up to 163840 entries are read once; longer rows twice.
 * A row outside every sample (a cu_seqlens that does not cover [0, T)) gets weight 0.
 * The loss is summed in a fixed order (bit-stable).  Asynchronous on `stream`; allocates nothing.
 * Errors: HBP_ERR_INVALID_ARG (NULL pointers, negative sizes, bad normaliser, t_ave <= 0 for
 * HBP_LOSS_STABLE), HBP_ERR_WORKSPACE, HBP_ERR_DEVICE.  total_tokens = 0 writes loss 0.
 */
hbp_status hbp_packed_ce(const void* logits, int64_t logit_stride_t, int32_t total_tokens, int32_t vocab,
                         const int32_t* labels, const int32_t* cu_seqlens, int32_t n_samples,
                         int32_t normalizer, float t_ave, void* dlogits_or_null, float* loss_out,
                         float* token_loss_or_null, void* workspace, size_t workspace_bytes, void* stream);

/*
 * hbp_mfma_probe — measurement aid: the second denominator of the roofline.  Launches, on `stream`,
 * one kernel in which every SIMD of `n_cu` compute units (two wavefronts each) issues nothing but
 * independent 32x32x16 bf16 MFMAs on register-resident data: `mfma_per_wave` of them per wavefront
 * (rounded down to a multiple of 4).  The caller times the launch (events on the same stream);
 * executed flops = n_cu * 8 * mfma_per_wave * 32768.  The operands are pseudo-random bf16 values of
 * magnitude 0.5 .. 1 with random signs (with constants the part clocks higher and the figure comes out
 * about a fifth larger).  That rate is what the matrix pipes of this part sustain under its power
 * limit on such data, i.e. the practical ceiling next to the published peak.
 * `sink` (device, >= n_cu * 512 floats) receives one value per thread so the work is not removed;
 * it carries no information.  Returns HBP_ERR_INVALID_ARG for NULL sink, n_cu < 1 or
 * mfma_per_wave < 4, HBP_ERR_DEVICE if the launch fails.  Asynchronous; allocates nothing.
 */
hbp_status hbp_mfma_probe(int32_t n_cu, int32_t mfma_per_wave, float* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* HBP_H */
