/*
 * ckv - Crystal-KV decode hot path for MI355X (gfx950): C ABI.
 *
 * One "unit" is the KV cache of one (layer, sequence, KV head).  Per decode
 * step and unit the library appends the new (k, v), computes GQA decode
 * attention over the unit's budgeted cache, updates every entry's LRFU score
 * (CRF) from the attention weights, and, when asked, evicts the lowest-score
 * entries down to the unit's budget and compacts the cache in place.  A
 * separate call re-allocates the budgets across layers and heads.
 * (arxiv 2601.16986: Sec. 2.2 attention; Sec. 5.2 and Alg. 1 attention-based
 * LRFU; Sec. 5.3 and Alg. 2 adaptive budget allocation; Sec. 3 answer-probe
 * classes.)
 *
 * Conventions
 *  - Every call returns 0 (CKV_OK) or a negative CKV_E* code; nothing throws
 *    or aborts across this boundary.  ckv_last_error() gives detail.
 *  - "dev" pointers are device (HBM) addresses, "host" pointers are ordinary
 *    host memory.  All device buffers are owned by the caller and must stay
 *    valid until ckv_destroy(); the library allocates no device memory.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls that take a stream only enqueue work on it and return; argument
 *    errors are reported synchronously, device-side conditions (a full cache
 *    at append) through ckv_status().  Calls documented as "synchronous" wait
 *    for the stream/device themselves.
 *  - A context is not thread safe.  All work of one context must be enqueued
 *    on streams that the caller orders; the usual case is a single stream.
 *  - Unit order everywhere: [layer][sequence][kv_head], C order.
 *  - Time: t is the position of the token being decoded; it starts at
 *    ckv_lrfu_params.t0 and advances by one when a decode step has covered
 *    the last layer.  t lives in device memory so that captured HIP graphs of
 *    decode steps can be replayed.
 */
#ifndef CKV_H
#define CKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ckv_ctx ckv_ctx;

enum {
  CKV_OK = 0,
  CKV_EINVAL = -1,     /* bad geometry, NULL pointer, parameter out of range */
  CKV_ECAPACITY = -2,  /* an append found a unit full (the caller skipped eviction) */
  CKV_ESTATE = -3,     /* call not valid in the context's current state */
  CKV_EHIP = -4,       /* a HIP runtime call or kernel launch failed */
  CKV_EWORKSPACE = -5  /* workspace too small or misaligned */
};

enum { CKV_BF16 = 1, CKV_F32 = 2 };                 /* out_dtype */
enum { CKV_REWARD_TOPP_HIT = 0,                      /* Alg. 1: reward 1 for entries in the top-p hit set */
       CKV_REWARD_ATTN_WEIGHTED = 1 };               /* variant: reward = mean attention weight, every entry stored */
enum { CKV_FLAG_HIT = 1,                             /* per-slot flag as exported: entry was in the last step's hit set */
       CKV_FLAG_SLIP = 2 };                          /* per-slot flag: slot holds the position of an entry evicted by the last eviction */
enum { CKV_CLASS_SLIP = 0, CKV_CLASS_POTENTIAL = 1, CKV_CLASS_CRYSTAL = 2 };

#define CKV_FUSE_EVICT 1u   /* ckv_decode_step: run Alg. 1 Step 4 in the same pass */
#define CKV_ATTENTION_ONLY 2u /* ckv_decode_step: append and attend only (the FullKV baseline of Table 1): no hit
                               * mask, no score update, no eviction; excludes CKV_FUSE_EVICT */
#define CKV_DEFER_BOOKKEEPING 4u /* ckv_decode_step of a single layer: only the attention output is ordered on the
                                  * caller's stream; scores and eviction follow on streams of the context (see there) */

/* Geometry.  head_dim must be 128; n_q_heads = G * n_kv_heads with G <= 8.
 * `cap` = the most entries a unit can ever hold, a multiple of 32, at most 32768.
 * Pool memory is handed to units in segments of 256 slots.  headroom = 0: every unit owns
 * ceil(cap / 256) segments for good (pool_slots >= units * ceil(cap / 256) * 256).  headroom = h >= 1:
 * the pools are shared, a unit owns the segments that budget + h entries need (h = the entries a unit may
 * hold above its budget between evictions: 1 when every step evicts), the rest is spare; segments move
 * between units and the spare list when budgets change (ckv_rebudget, ckv_set_budgets) or a prompt longer
 * than the budget passes through (ckv_load_prompt), see ckv_rebalance.  ckv_pool_slots gives the need. */
typedef struct {
  int32_t n_layers, batch, n_q_heads, n_kv_heads, head_dim;
  int32_t cap;
  int32_t out_dtype;      /* CKV_F32 or CKV_BF16: element type of `out` in ckv_decode_step */
  int32_t headroom;
  int64_t pool_slots;     /* slots in each pool, a multiple of 256 */
} ckv_layout;

/* Parameters of Alg. 1 / Alg. 2 (Sec. 6.4 recommends top_p = 0.9, lambda in [0.5, 0.7]). */
typedef struct {
  float lambda;           /* CRF decay, in [0, 1]; 0^0 = 1 */
  float top_p;            /* hit-mask threshold p > 0 of Alg. 1 Step 1; >= 1 marks every entry */
  float softmax_scale;    /* multiplies q.k before the softmax (1/sqrt(head_dim) usually) */
  int32_t reward_mode;    /* CKV_REWARD_* */
  int32_t t0;             /* time of the first decode step = number of prompt positions */
  int32_t budget_min;     /* bounds for budgets, 1 <= budget_min <= budget_max < cap */
  int32_t budget_max;
} ckv_lrfu_params;

/* Caller-owned device buffers.  With S = ckv_layout.pool_slots:
 *   k_pool, v_pool : S * 128 bf16 each, in segments of 256 slots (64 KB).  Which
 *                    segments hold a unit's entries, in which order, is recorded
 *                    in the segment table in the workspace (ckv_get_segments).
 *                    Inside a segment, entries are stored in blocks of 32 entries
 *                    (8 KB) in a tiled order chosen so that a 64-lane wavefront
 *                    reads 1 KB contiguous per load and gets MFMA operands
 *                    directly; use ckv_load_prompt / ckv_import_unit /
 *                    ckv_export_unit to convert from and to row-major.
 *   crf  : S float   - stored CRF score of each slot
 *   tau  : S int32   - time the stored CRF refers to (last hit)
 *   pos  : S int32   - position of the token the slot's entry came from
 *   flags: S uint8   - CKV_FLAG_SLIP marks.  The hit mark is not stored per
 *                      step: in the top-p mode an entry was hit in its unit's
 *                      last step iff its tau equals that step's time;
 *                      ckv_export_unit adds CKV_FLAG_HIT accordingly.
 *   workspace : ckv_workspace_bytes() bytes, 256-byte aligned.
 * ckv_init overwrites all of them. */
typedef struct {
  void* k_pool;
  void* v_pool;
  float* crf;
  int32_t* tau;
  int32_t* pos;
  uint8_t* flags;
  void* workspace;
  size_t workspace_bytes;
} ckv_buffers;

/* Bytes of workspace ckv_init needs for this geometry and these parameters
 * (0 if they are invalid). */
size_t ckv_workspace_bytes(const ckv_layout* layout, const ckv_lrfu_params* params);

/* Create a context.  `budgets` is a host array [n_layers][batch][n_kv_heads]
 * with budget_min <= B <= budget_max; each sequence's total is what Alg. 2
 * later conserves (B_total).  Clears the pools and the per-unit state on
 * `stream` and waits for it (synchronous).  Errors: CKV_EINVAL, CKV_EWORKSPACE,
 * CKV_EHIP. */
int ckv_init(ckv_ctx** ctx, const ckv_layout* layout, const int32_t* budgets,
             const ckv_lrfu_params* params, const ckv_buffers* buffers, void* stream);

/* Release host-side state.  Device buffers stay the caller's. */
void ckv_destroy(ckv_ctx* ctx);

/* Fill the empty caches of one layer with a prompt.  k, v: dev bf16
 * [batch][n_kv_heads][P][128] row-major; entries get positions 0..P-1.
 * crf0 / tau0: dev [batch][n_kv_heads][P] or NULL (then CRF = 1, tau = P-1:
 * referenced once, at the end of the prompt; the paper is silent on prompt
 * scores).  Requires 0 < P < cap, P <= t0 and the layer's units empty
 * (CKV_ESTATE otherwise).  With shared pools the layer's units first get the
 * segments that P + headroom entries need from the spare list (see
 * ckv_rebalance); a unit for which they are not there is loaded as far as it has
 * room, and ckv_status() reports CKV_ECAPACITY. */
int ckv_load_prompt(ckv_ctx* ctx, int32_t layer, const void* k, const void* v, int32_t P,
                    const float* crf0, const int32_t* tau0, void* stream);

/* Scores of a loaded prompt from its last W queries (the step before the decode
 * path: Alg. 1 Steps 1-3, Sec. 5.2, replayed; the paper does not say what scores
 * the prompt's entries start with).  q_obs: dev bf16 [W][batch][n_q_heads][128],
 * the queries of positions P-W .. P-1 in order.  Replaces the CRF and tau the
 * layer's prompt was loaded with: every entry starts as referenced once, on
 * arrival (CRF 1, tau = position), then for t = P-W .. P-1 the query of position
 * t attends to the entries of positions <= t and their scores are updated at
 * time t exactly as in a decode step that evicts nothing, position t's own
 * entry being in its hit set.  Nothing is appended, evicted or written to an
 * output, the time stays t0, and the replay leaves no trace in the aggregated
 * CRF that ckv_rebudget consumes.  Requires a layer filled by ckv_load_prompt
 * and not touched since (CKV_ESTATE otherwise) and 1 <= W <= P.  The keys are read
 * twice per batch of queries (up to 16 floor(16 / G) of them, G = n_q_heads /
 * n_kv_heads; fewer when the workspace of a context with few layers holds less),
 * the values not at all (only weights are needed); the workspace's logits and
 * partials of the decode paths serve as scratch (their contents are dead between
 * calls).  Five kernel launches per batch plus two on `stream`; asynchronous. */
int ckv_seed_prompt(ckv_ctx* ctx, int32_t layer, const void* q_obs, int32_t W, void* stream);

/* Fill the empty caches of one layer with entries from the middle of a
 * sequence (restoring a checkpoint, or building a steady-state cache for
 * measurements).  k, v as in ckv_load_prompt with row stride P; unit (b, h)
 * takes its first lengths[b][h] rows (dev int32 [batch][n_kv_heads], NULL = P);
 * pos0: dev int32 [batch][n_kv_heads][P], the entries' positions, which must be
 * distinct within a unit and below the current time (NULL = 0..P-1); crf0 /
 * tau0 as in ckv_load_prompt.  Nothing about the values is checked. */
int ckv_load_cache(ckv_ctx* ctx, int32_t layer, const void* k, const void* v, int32_t P,
                   const int32_t* lengths, const float* crf0, const int32_t* tau0, const int32_t* pos0,
                   void* stream);

/* One decode step (Sec. 2.2 + Alg. 1 Steps 1-3, optionally Step 4) for one
 * layer, or for all layers when layer == -1.
 *   q      : dev bf16 [batch][n_q_heads][128]   (leading [n_layers] if layer == -1)
 *   k_new,
 *   v_new  : dev bf16 [batch][n_kv_heads][128]  (same)
 *   out    : dev out_dtype [batch][n_q_heads][128] (same) - softmax(scale q K^T) V
 * Appends (k_new, v_new) at position t (CRF 0, tau t), attends over the unit's
 * entries, takes the mean weight over the G query heads of each KV head,
 * builds the top-p hit set (the new entry always belongs to it), updates the
 * hit entries' stored CRF and tau (tau = t marks the hit), accumulates the unit's
 * aggregated CRF for Alg. 2, and with CKV_FUSE_EVICT evicts down to the budget
 * (as ckv_evict).  Layers must be stepped in order 0..n_layers-1; t advances
 * after the last one.  A unit that is already full (n == cap, or with shared
 * pools n == 256 * the segments it owns) is not appended to: the step still
 * runs and ckv_status() reports CKV_ECAPACITY.
 * With CKV_ATTENTION_ONLY the stored scores, taus and the Alg. 2 window are left
 * alone (the new entry is still appended with CRF 0, tau t).
 * With CKV_DEFER_BOOKKEEPING (single-layer calls only) the call puts on `stream`
 * only what the next operation of a model needs: one kernel that attends over the
 * cache and the new entry and writes the output (and the new entry's rows into
 * the cache).  The append's records, the hit set, the scores and the eviction of
 * that layer follow on one of two streams the context owns, up to eight
 * consecutive layers per launch, beside whatever `stream` does next (the next
 * layers' steps, the model's other work).  Results are the same up to
 * floating-point summation order.  (A layer with at least two units per compute
 * unit is finished sooner by the fused kernel, bookkeeping included: there the
 * flag has no effect.)  Every later
 * ckv_* call that takes a stream orders itself after the bookkeeping it depends
 * on (the next step of the same layer after that layer's, everything else after
 * all of it); the host-side getters wait for the whole device.  ckv_join orders
 * a stream after all of it explicitly: call it before reading the caller-owned
 * state arrays directly, and before ending a stream capture that contains such
 * steps (the context's streams take part in the capture and must rejoin it). */
int ckv_decode_step(ckv_ctx* ctx, int32_t layer, const void* q, const void* k_new,
                    const void* v_new, void* out, uint32_t flags, void* stream);

/* Alg. 1 Step 4 for every unit of `layer` (-1: all) holding more entries than
 * its budget B: keep the B entries that come first by (CRF_temp descending,
 * position ascending), where CRF_temp is the score decayed to the unit's last
 * decode step; move survivors into slots [0, B) (slot order is unspecified);
 * slots [B, n_old) then hold the evicted positions with CKV_FLAG_SLIP. */
int ckv_evict(ckv_ctx* ctx, int32_t layer, void* stream);

/* A comparison policy on the same caches, not part of the method (Sec. 2.3: the
 * baseline that assumes attention goes to the initial and the most recent
 * tokens).  For every unit of `layer` (-1: all) holding more entries than its
 * budget B: keep the entries whose position is below n_sink (the lowest of them
 * if even they exceed B) and fill the budget with the highest positions; scores
 * play no part and stay as they are on the survivors.  Slots, flags and the
 * eviction record as after ckv_evict.  n_sink < 0: CKV_EINVAL. */
int ckv_evict_window(ckv_ctx* ctx, int32_t layer, int32_t n_sink, void* stream);

/* Alg. 2: new integer budgets for every (layer, head) of every sequence from
 * the aggregated CRF averaged over the decode steps since the last call (or
 * since init), keeping each sequence's total; restarts the averaging window.
 * Budgets stay within [budget_min, budget_max].  No entries move: the next
 * eviction brings units down to shrunken budgets. */
int ckv_rebudget(ckv_ctx* ctx, void* stream);

/* Shared pools (headroom >= 1) only; a no-op otherwise.  Deals the pool segments out again: every unit ends up
 * owning what max(budget + headroom, its entries) needs, surplus goes to the spare list first, deficits are
 * served from it in unit order (deterministic).  The library calls this by itself: inside ckv_load_prompt and
 * ckv_load_cache (the layer's units get room for the P entries and an append), and at the start of the first
 * decode step (layer 0 or all layers) after an eviction that covered the last layer (a decode step with
 * CKV_FUSE_EVICT, ckv_evict, ckv_evict_window) once budgets have changed (ckv_rebudget, ckv_set_budgets) or a
 * prompt has passed through - not right behind that eviction, so that the record of what a unit evicted (the
 * slots behind its entries) can still be exported.  Between a budget change and that point a grown unit still
 * fits: it has room for headroom entries above its old budget.  If the spare list is short nobody is given anything and
 * ckv_status() reports CKV_ECAPACITY; a unit that owns too little refuses appends the same way.
 * Asynchronous on `stream`; one 1024-thread workgroup. */
int ckv_rebalance(ckv_ctx* ctx, void* stream);

/* Slots each pool needs (a multiple of 256; 0 on bad arguments).  headroom 0: units * ceil(cap / 256) * 256.
 * Shared pools: what the budgets' total plus headroom per unit needs, one segment per unit on top (the most
 * that rounding to segments can waste, however Alg. 2 redistributes the budgets), plus, if prompt_len > 0,
 * one layer's units at prompt_len + headroom entries (a prompt on its way through ckv_load_prompt,
 * ckv_seed_prompt and ckv_evict while the other layers sit at their budgets).  Host budgets as in ckv_init. */
int64_t ckv_pool_slots(const ckv_layout* layout, const int32_t* budgets, int32_t prompt_len);

/* Sec. 3 answer-probe classes for one layer: attention of `q_probe` (dev bf16
 * [batch][n_q_heads][128]) over the current caches, no state change; per slot
 * class (CKV_CLASS_*) written to classes (dev uint8, [batch][n_kv_heads][cap]):
 * top floor(0.3 n) by (mean weight descending, position ascending) Crystal,
 * last floor(0.3 n) Slip, the rest Potential. */
int ckv_probe(ckv_ctx* ctx, int32_t layer, const void* q_probe, uint8_t* classes, void* stream);

/* ckv_probe for callers that cannot allocate or bring a workspace of their own for it: code under HIP graph
 * capture, tight serving loops that probe beside decode steps, harnesses that forbid hipMalloc.  Same
 * arguments, same result (the classes are identical, byte for byte), but the scan's scratch - work list,
 * partial results, logits, launch counters - lives in a static device array of 128 MiB that the library
 * owns on every GPU it is loaded on (held until the process ends), not in the context's workspace; so the
 * call leaves the context's workspace alone.  It calls no hipMalloc, hipFree or
 * other allocating routine.  A layer whose scratch (about batch * n_kv_heads * cap * 6 * G bytes, G = n_q_heads / n_kv_heads) does
 * not fit is refused with CKV_EWORKSPACE; a context created on another device than the current one, or a
 * per-layer step in progress, with CKV_ESTATE.  All calls on one GPU share the array, whose contents
 * persist from call to call: calls that overlap on one GPU (two streams, two contexts, two threads) race;
 * calls ordered on one stream, or by events, do not.  Asynchronous on `stream`. */
int ckv_probe_noalloc(ckv_ctx* ctx, int32_t layer, const void* q_probe, uint8_t* classes, void* stream);

/* Synchronous readers (wait for the device). Host arrays [n_layers][batch][n_kv_heads]. */
int ckv_get_budgets(ckv_ctx* ctx, int32_t* budgets);
int ckv_get_lengths(ckv_ctx* ctx, int32_t* lengths);
int ckv_set_budgets(ckv_ctx* ctx, const int32_t* budgets);   /* same checks as ckv_init; B_total recomputed */
/* The segment table: owned[units] = segments each unit owns, rows[units][ceil(cap / 256)] = their pool indices
 * in order (0 in the columns behind them), spare[pool_slots / 256] = the first *n_spare entries are the pool
 * segments nobody owns.  owned, rows and spare may be NULL. */
int ckv_get_segments(ckv_ctx* ctx, int32_t* owned, int32_t* rows, int32_t* spare, int32_t* n_spare);
int ckv_get_time(ckv_ctx* ctx, int32_t* t);
int ckv_set_time(ckv_ctx* ctx, int32_t t);                   /* also restarts the Alg. 2 window */
/* CKV_OK; CKV_ECAPACITY if, since the last call, some append found its unit full or the spare list ran short when
 * pool segments were dealt out; CKV_EHIP if a bounded wait inside a kernel gave up (results invalid).  Reported once. */
int ckv_status(ckv_ctx* ctx);

/* Synchronous state transfer of one unit, row-major on the host side (tests,
 * checkpointing).  Export: *n entries, *n_evicted log slots after them; the
 * host arrays must hold `cap` slots (K, V: cap*128 bf16 as uint16).  Any
 * output pointer may be NULL; slots in segments the unit does not own read as
 * zero.  Import: replaces the unit's entries (n < cap, and with shared pools
 * n < 256 * the segments the unit owns: CKV_ECAPACITY otherwise) and sets its
 * last-step time to t_unit. */
int ckv_export_unit(ckv_ctx* ctx, int32_t layer, int32_t seq, int32_t head, int32_t* n,
                    int32_t* n_evicted, int32_t* budget, uint16_t* K, uint16_t* V, float* crf,
                    int32_t* tau, int32_t* pos, uint8_t* flags);
int ckv_import_unit(ckv_ctx* ctx, int32_t layer, int32_t seq, int32_t head, int32_t n,
                    const uint16_t* K, const uint16_t* V, const float* crf, const int32_t* tau,
                    const int32_t* pos, int32_t t_unit);

/* Timing hook for benchmarks: while enabled, every ckv_decode_step brackets
 * its dominant kernel (the fused per-unit kernel, or the scan kernel when the
 * separate kernels are used) with HIP events on the launch stream (do not
 * enable while the stream is being captured into a graph).  ckv_profile_read
 * waits for the device and returns that kernel's summed time and launch count
 * since enabling. */
int ckv_profile_enable(ckv_ctx* ctx, int32_t on);
int ckv_profile_read(ckv_ctx* ctx, double* scan_ms, int32_t* launches);

/* Which kernels ckv_decode_step uses: 0 = choose by unit count (default),
 * 1 = separate scan and finish kernels, 2 = the fused per-unit kernel, which
 * keeps the logits in LDS, in the widest variant that fits; 3 / 4 = the fused
 * kernel with 4 / 2 wavefronts per unit (2 / 4 workgroups per compute unit).
 * Whatever the mode, a single-layer call takes the separate kernels if the
 * layer has fewer units than the fused kernel has workgroups or if its
 * bookkeeping is deferred.  A variant needs 4 * cap
 * bytes of LDS in its workgroup's share (CKV_EINVAL otherwise).  Results do not depend on the choice beyond
 * floating-point summation order.
 * ckv_path_info reports what all-layer steps use under the current mode:
 * *fused_waves = wavefronts per unit of the fused variant (0: separate
 * kernels), *lds_main_bytes = bytes of its LDS tile for logits and per-entry
 * values. */
int ckv_set_path(ckv_ctx* ctx, int32_t mode);
int ckv_path_info(ckv_ctx* ctx, int32_t* fused_waves, int32_t* lds_main_bytes);

/* Orders `stream` after the bookkeeping that steps with CKV_DEFER_BOOKKEEPING have
 * left in flight on the context's own streams (no-op if there is none). */
int ckv_join(ckv_ctx* ctx, void* stream);

/* Measurement aid, independent of any context: streams `bytes` (a multiple of
 * 16 KiB is read completely; at least 1 MiB) from dev `src` with plain 16-byte
 * non-temporal loads (dst == NULL; `sink` is a dev uint32 that is never
 * actually written) or copies them to dev `dst`.  Gives the on-box bandwidth
 * ceiling next to which the streaming kernels are reported, and kernels of known size
 * for calibrating profiler byte counters.  Pointers 16-byte aligned. */
int ckv_bandwidth_probe(const void* src, void* dst, size_t bytes, void* sink, void* stream);

const char* ckv_strerror(int code);
const char* ckv_last_error(const ckv_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* CKV_H */
