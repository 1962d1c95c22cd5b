/*
 * odc.h -- C ABI of the MI355X (gfx950) library for the data-parallel hot path of
 * On-Demand Communication (ODC), "Revisiting Parameter Server in LLM Post-Training".
 *
 * The paper (Section 3) replaces FSDP's per-layer collectives by two point-to-point
 * primitives: gather (a worker fetches every owner's parameter shard and so obtains the
 * full layer, in place of all-gather) and scatter-accumulate (a worker pushes slice r of
 * its gradient to owner r, who adds it to its gradient shard, in place of reduce-scatter;
 * Appendix B: the owner accumulates each contribution when it arrives).  Parameters and
 * gradients are partitioned evenly over the R devices (Section 3.1) in FSDP's flat memory
 * layout, and the accumulated gradients are read at the minibatch end (Section 3.2).
 *
 * In this library one GPU holds every logical rank's shard as a separate HBM buffer and
 * executes all R owners' copies and accumulations itself: no peer access, no collectives.
 *
 * Conventions for every entry point
 *   - All element data live in DEVICE memory owned by the caller.  Parameters and
 *     gradient contributions are bf16 (raw 16-bit patterns); accumulators are IEEE-754
 *     binary32.  Pointer arrays of length R ("[R] host") are HOST arrays of device
 *     pointers; the library copies them during the call and keeps no reference.
 *   - Every device base pointer (each shard, the full buffer, each accumulator shard, the
 *     gradient) must be 16-byte aligned, else ODC_ERR_ALIGNMENT.  Interior boundaries
 *     (r * S_t) may fall anywhere; that is the library's business.  The kernels are
 *     fastest when the bases are 128-byte aligned (a wavefront then writes whole cache
 *     lines), which device allocators give anyway.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Launch
 *     calls only enqueue work on it and return: they never synchronise the device and never
 *     allocate or free device memory.  On the host, the ordered mode takes the layout's mutex
 *     for the duration of the call and, the first time it sees an accumulator set, allocates
 *     one small bookkeeping node (see ODC_ORDERED below); odc_reduce_groups sorts a temporary
 *     host copy of its R output pointers; nothing else allocates.
 *     A call enqueues one kernel per group of up to 64 ranks, so exactly one kernel for
 *     R <= 64, for any number of tensors T.  With R > 64, if a later group's launch fails
 *     (ODC_ERR_HIP) the earlier groups' kernels are already enqueued: the accumulators are then
 *     partly updated, and the contribution counts as issued.
 *   - Return value: ODC_OK (0) or a negative ODC_ERR_* code.  All argument errors are
 *     detected on the host before anything is enqueued.  Nothing throws or aborts.
 *   - Padding (shard slots whose flat index is >= numel) and the alignment gaps between tensors
 *     never reach a result and never change, by any call.  The read-modify-write calls
 *     (scatter-accumulate, its fused form, the staging drain) may load such a slot together
 *     with the valid slots of its 16-byte vector and store the very same bits back, so that
 *     cache lines are written whole; every other call does not touch them at all.
 */
#ifndef ODC_H
#define ODC_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct odc_layout odc_layout_t; /* opaque; owned by the library */

#define ODC_OK 0
#define ODC_ERR_INVALID_ARG (-1) /* null pointer, R/T/numel < 1, worker or microbatch out of range, bad flags */
#define ODC_ERR_ALIGNMENT (-2)   /* a device base pointer is not 16-byte aligned */
#define ODC_ERR_ORDER (-3)       /* ordered contribution not after the previous one for this accumulator set */
#define ODC_ERR_OVERFLOW (-4)    /* sizes do not fit 63-bit element or byte counts */
#define ODC_ERR_HIP (-5)         /* a HIP call failed; see odc_last_hip_error() */
#define ODC_ERR_NO_DEVICE (-6)   /* layout was built host-only, or belongs to another device */
#define ODC_ERR_NOMEM (-7)       /* host allocation failed */
#define ODC_ERR_TOO_LARGE (-8)   /* size beyond the fixed scratch of a no-allocation entry point */

#define ODC_MAX_RANKS 4096

/* odc_init_layout flags */
#define ODC_LAYOUT_HOST_ONLY 1 /* integer layout only: no HIP call is made, launches are refused */

/* odc_scatter_accumulate flags */
#define ODC_ORDERED 0   /* plain read-add-write; bit-exact if issued in (worker, microbatch) order on one stream */
#define ODC_UNORDERED 1 /* hardware float atomics; calls may be issued in any order and from several streams */

/*
 * Build the shard layout (Section 3.1: even partition over R owners; FSDP flat-param
 * layout, Section 3) for T flat parameters of numel[t] >= 1 elements.
 *   S_t          = ceil(numel[t] / R)                 slots of tensor t in every owner's shard
 *   owner r      holds flat indices [r*S_t, (r+1)*S_t) of tensor t; indices >= numel[t] are padding
 *   valid(t, r)  = clamp(numel[t] - r*S_t, 0, S_t)
 * Buffer placement chosen by the library: inside an owner's buffer ("rank arena") and inside
 * the full-length buffer, tensor t starts at a multiple of 8 elements (16 bytes of bf16)
 * after tensor t-1; see odc_shard_offset / odc_full_offset.  For T = 1 both offsets are 0,
 * a rank arena is exactly S_0 slots and the full buffer exactly numel[0] elements.
 * Unless ODC_LAYOUT_HOST_ONLY is set, a descriptor table is allocated with hipMalloc on the
 * current device (this call may synchronise); the layout can then be used on that device only.
 * numel is a host array, copied.  *out receives the handle; free it with odc_free_layout.
 */
int odc_init_layout(int R, int T, const int64_t *numel, int flags, odc_layout_t **out);

/* Release a layout and its device table (NULL is ignored).  Do not call while kernels that
 * use the layout may still be running. */
void odc_free_layout(odc_layout_t *layout);

/* Layout queries (host, pure).  Return -1 for a NULL layout or an index out of range. */
int odc_num_ranks(const odc_layout_t *layout);
int odc_num_tensors(const odc_layout_t *layout);
int64_t odc_numel(const odc_layout_t *layout, int t);
int64_t odc_shard_elems(const odc_layout_t *layout, int t);        /* S_t */
int64_t odc_valid_elems(const odc_layout_t *layout, int t, int r); /* valid(t, r) */
int64_t odc_rank_arena_elems(const odc_layout_t *layout);          /* elements each owner buffer must hold */
int64_t odc_full_elems(const odc_layout_t *layout);                /* elements the full-length buffer must hold */
int64_t odc_shard_offset(const odc_layout_t *layout, int t);       /* start of tensor t inside a rank arena */
int64_t odc_full_offset(const odc_layout_t *layout, int t);        /* start of tensor t inside the full buffer */

/*
 * Gather (Section 3; Appendix B: each rank pulls the shards of all ranks):
 *   full_out[full_off_t + r*S_t + i] = param_shards[r][shard_off_t + i]   for i < valid(t, r)
 * bits copied unchanged.
 *   param_shards  [R] host array of device pointers, bf16, each >= odc_rank_arena_elems elements, read only
 *   full_out      device, bf16, >= odc_full_elems elements; only valid elements are written
 * Algorithmic HBM traffic: 4 bytes per valid element.
 */
int odc_gather(const odc_layout_t *layout, const void *const *param_shards, void *full_out,
               void *stream);

/*
 * One scatter-accumulate contribution (Section 3; Appendix B; Section 2.1 with w_m = 1):
 * worker `worker`'s gradient for its microbatch `microbatch`, laid out like the full
 * buffer, is cut into R slices and slice r is added into owner r's accumulator:
 *   accum_shards[r][shard_off_t + i] += widen(grad_full[full_off_t + r*S_t + i])   for i < valid(t, r)
 * widen(bf16) is exact; the sum is one binary32 addition, round-to-nearest-even, subnormals kept.
 *   grad_full     device, bf16, >= odc_full_elems elements, read only
 *   accum_shards  [R] host array of device pointers, binary32, each >= odc_rank_arena_elems elements
 *   worker        in [0, R); microbatch >= 0
 *   flags         ODC_ORDERED: the result is bit-identical to the sequential sum in
 *                 (worker, microbatch) lexicographic order provided the caller issues the
 *                 contributions of one accumulator set in that order on one stream.  The library
 *                 remembers the last (worker, microbatch) per (layout, accum_shards[0]) and
 *                 returns ODC_ERR_ORDER, enqueuing nothing, if a call is not strictly later;
 *                 odc_reset_accum and odc_forget_accum forget it, and so does freeing the
 *                 layout.  The table holds at most 1024 accumulator sets per layout; beyond
 *                 that the least recently used entry is dropped (that set then starts afresh).
 *                 The key is an address: accumulators that are freed without a reset and whose
 *                 address is handed out again would inherit the old history -- call
 *                 odc_forget_accum (or odc_reset_accum) before freeing or after reallocating.
 *                 Two ordered calls on the same accumulators
 *                 running concurrently on different streams race (caller error).
 *                 ODC_UNORDERED: each element is added with a device-scope float atomic add
 *                 (no order check); concurrent calls on several streams are safe, the result
 *                 depends on arrival order within the usual binary32 summation error, and the
 *                 atomic unit may flush subnormal values to zero.
 * Algorithmic HBM traffic: 10 bytes per valid element (2 + 4 read, 4 written).
 */
int odc_scatter_accumulate(const odc_layout_t *layout, const void *grad_full,
                           void *const *accum_shards, int worker, int microbatch, int flags,
                           void *stream);

/*
 * Weighted contribution (Section 2.1: the accumulated gradient is the sum of w_m * g^(m), with
 * w_m = 1 for a plain sum or a token- or sample-proportional weight for an average).  Same
 * arguments, ordering rules and history as odc_scatter_accumulate, plus `weight`:
 *   accum_shards[r][shard_off_t + i] = fma32(weight, widen(grad_full[...]), accum_shards[r][...])
 * one fused multiply-add per element, i.e. a single rounding of weight*g + acc (the paper does
 * not fix the rounding; this is the reading taken).  With weight = 1 the result is that of
 * odc_scatter_accumulate bit for bit.  ODC_UNORDERED rounds the product first and adds it
 * atomically.  Algorithmic HBM traffic: 10 bytes per valid element.
 */
int odc_scatter_accumulate_weighted(const odc_layout_t *layout, const void *grad_full,
                                    void *const *accum_shards, int worker, int microbatch,
                                    float weight, int flags, void *stream);

/*
 * Fused form of odc_scatter_accumulate for an owner that finds several contributions staged
 * at once (Appendix B gives every client its own receive buffer, so up to one contribution
 * per client can be waiting): `count` gradients are applied in the given order in ONE pass,
 *   acc = (((acc + g_0) + g_1) + ... + g_{count-1})
 * the same left-to-right binary32 sequence that `count` single calls perform, so in
 * ODC_ORDERED mode the result is bit-identical to theirs, while the accumulators are read
 * and written once: (2*count + 8) bytes per valid element instead of 10*count.
 *   count         1 .. ODC_MAX_FUSED
 *   grads         [count] host array of device pointers (bf16, full layout, 16-byte aligned)
 *   workers, microbatches  [count] host arrays; in ODC_ORDERED mode strictly ascending
 *                 (worker, microbatch) pairs, the first one after this accumulator set's history
 *                 (ODC_ERR_ORDER otherwise, nothing enqueued); the history becomes the last pair.
 *   ODC_UNORDERED sums the count values in registers as a balanced binary tree (pairwise) and
 *                 issues one atomic add per element: C contributions taken `count` at a time pass
 *                 through ceil(log2 count) + ceil(C / count) roundings instead of C.
 */
#define ODC_MAX_FUSED 8
int odc_scatter_accumulate_multi(const odc_layout_t *layout, int count, const void *const *grads,
                                 void *const *accum_shards, const int *workers, const int *microbatches,
                                 int flags, void *stream);

/*
 * Server-side staging (Appendix B).  Every owner keeps one receive buffer per client -- M/N
 * elements each, M per owner, where M is the layer size and N the number of devices -- because
 * several clients may push at once while one client's requests are serialised.  A push writes
 * the worker's slice into its slot of every owner's buffer and then signals the owner; the
 * owner's daemon accumulates whatever has arrived.  Here the signal is a device-side flag and
 * the daemon's polling loop becomes odc_stage_drain, which handles what is there and returns
 * (no kernel ever waits).
 *
 *   staging_shards [R] host array of device pointers: owner r's buffer, bf16, R slots of
 *                  odc_stage_slot_elems() elements (the rank arena rounded up to a multiple of
 *                  64 elements; client w's slot starts at w * slot and mirrors the rank arena;
 *                  what a slot holds outside the valid elements of its pieces is unspecified
 *                  and never used); 16-byte aligned, fastest when 128-byte aligned
 *   flags          device int32[odc_stage_flag_count()] = R*R slot states (owner-major: owner r,
 *                  client w at r*R + w; 0 empty, 1 full, 2 being written) + 1 counter of refused pushes
 *   snapshot       device int32[odc_stage_snapshot_count()], scratch owned by the caller; a
 *                  drain writes and reads it, so two drains that overlap must not share one
 *
 * odc_stage_init   zeroes flags (a small fill kernel on `stream`).
 * odc_stage_push   decides ONCE per owner, before any byte is copied, whether the owner takes the
 *                  push: slot (r, worker) empty -> being written (an atomic compare-and-swap by
 *                  one thread).  Slice r of grad_full (full layout) is then copied into the
 *                  slots so claimed, and those become full.  An owner whose slot is not empty
 *                  refuses the whole push and is counted in flags[R*R]: a client has one buffer
 *                  per owner, so it must not push again before the owner has drained.
 *                  4 bytes per valid element.
 * odc_stage_drain  takes one snapshot of the slots that are full (never one that is being
 *                  written); every owner with full slots reads and writes its accumulator once
 *                  and adds the staged slices in ascending client order,
 *                  acc = (((acc + s_w1) + s_w2) + ...), one binary32 add each -- the same bits as
 *                  single ordered contributions in that order; then empties exactly the slots
 *                  of the snapshot.  Owners with nothing staged are not touched.
 *                  (2k + 8) bytes per valid element for k staged slices.
 * All three enqueue on `stream` and return.  Pushes and drains on one stream are ordered by
 * it.  A push may run concurrently with a drain on another stream, however their kernels
 * interleave: per owner the push is either refused as a whole (its slot was not empty when it
 * was claimed) or taken as a whole and added by exactly one drain -- the one running, if its
 * snapshot came after the push had finished, else the next.  Every flag access is a
 * device-scope atomic with acquire/release ordering.  What the caller must serialise: the
 * pushes of one client (one stream per client will do), and the drains of one staging set.
 * If a push returns ODC_ERR_HIP some of its slots may be left in the "being written" state:
 * call odc_stage_init again before reusing the staging set.  The ordered-mode history of
 * odc_scatter_accumulate is not involved: the order is the drain order.
 */
int64_t odc_stage_slot_elems(const odc_layout_t *layout);
int64_t odc_stage_flag_count(const odc_layout_t *layout);
int64_t odc_stage_snapshot_count(const odc_layout_t *layout);
int odc_stage_init(const odc_layout_t *layout, void *flags, void *stream);
int odc_stage_push(const odc_layout_t *layout, const void *grad_full, void *const *staging_shards,
                   void *flags, int worker, void *stream);
int odc_stage_drain(const odc_layout_t *layout, const void *const *staging_shards, void *flags,
                    void *snapshot, void *const *accum_shards, void *stream);

/*
 * odc_stage_drain for callers that cannot allocate and have no workspace to hand over: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and
 * result as odc_stage_drain without `snapshot`: the snapshot list lives in a fixed device array
 * inside the library (ODC_NOALLOC_MAX_RANKS * (ODC_NOALLOC_MAX_RANKS + 1) int32 = 263,168
 * bytes, one copy per GPU the library runs on, held until the process ends).  The call
 * allocates and frees nothing, on the host or on the device.  Layouts with more than
 * ODC_NOALLOC_MAX_RANKS ranks are refused with ODC_ERR_TOO_LARGE, nothing enqueued.  All calls
 * on one GPU share the one array: calls that may overlap in time (different streams, or
 * different layouts on different streams) race on it -- serialise them, or use
 * odc_stage_drain with a workspace each.  Nothing needs clearing between calls: every drain
 * rewrites the part of the array it reads.
 */
#define ODC_NOALLOC_MAX_RANKS 256
int odc_stage_drain_noalloc(const odc_layout_t *layout, const void *const *staging_shards, void *flags,
                            void *const *accum_shards, void *stream);

/* odc_retrieve_grads output types */
#define ODC_OUT_F32 0
#define ODC_OUT_BF16 1

/*
 * Minibatch end (Section 3.2: the integration retrieves the accumulated gradients at the
 * minibatch end; each owner then holds what reduce-scatter would have left on it, Section 2.2).
 *   out_shards[r][shard_off_t + i] = cast(fl32(scale * accum_shards[r][shard_off_t + i]))   i < valid(t, r)
 * one binary32 multiplication (scale = 1 for a sum, 1/tokens or 1/samples for an average), then
 * no further rounding (ODC_OUT_F32, out_shards are binary32) or one rounding to nearest-even to
 * bf16 (ODC_OUT_BF16; NaN stays NaN).  The accumulators are not modified and the ordered-mode
 * history is kept; call odc_reset_accum before the next minibatch.
 *   accum_shards  [R] host array of device pointers, binary32, read only
 *   out_shards    [R] host array of device pointers, >= odc_rank_arena_elems elements each, 16-byte aligned
 * Algorithmic HBM traffic: 8 (binary32 out) or 6 (bf16 out) bytes per valid element.
 */
int odc_retrieve_grads(const odc_layout_t *layout, const void *const *accum_shards,
                       void *const *out_shards, float scale, int out_dtype, void *stream);

/*
 * Unordered accumulation with a guaranteed error: wide accumulators.  Contributions arrive in any
 * order (Appendix B: the owner accumulates on receipt while several clients push).  A binary32
 * accumulator updated one contribution at a time can be off by up to (C - 1) * 2^-24 * sum|g|
 * after C contributions whatever the order, which exceeds 1e-6 * sum|g| for C > 17 on inputs
 * built for it.  These calls keep the running sum in binary64 shards instead and round it to
 * binary32 once, at retrieval: the retrieved gradient is within 2^-24 * (1 + C * 2^-29) * sum|g|
 * (6e-8) of the exact sum for any inputs, any order, any number of streams.
 *   accum64_shards  [R] host array of device pointers, IEEE binary64, >= odc_rank_arena_elems
 *                   elements each (same element offsets as the binary32 accumulators), 16-byte aligned
 * odc_reset_accum_wide          every valid element becomes +0.0.  8 bytes per valid element.
 * odc_scatter_accumulate_wide   acc64[r][...] += widen(grad_full[...]) with one device-scope binary64
 *                               atomic add per valid element; no order, no history, safe from
 *                               several streams at once.  The atomics run at the memory side like the
 *                               binary32 ones of ODC_UNORDERED, at about half their element rate.
 * odc_retrieve_grads_wide       out_shards[r][...] = cast(fl32(scale * fl32(acc64[r][...]))): one
 *                               rounding to binary32, then the multiply and cast of
 *                               odc_retrieve_grads (out_dtype as there).  The accumulators are not
 *                               modified.  12 or 10 bytes per valid element.
 * Padding is never written.  All three enqueue one kernel per group of up to 64 ranks and return.
 */
int odc_reset_accum_wide(const odc_layout_t *layout, void *const *accum64_shards, void *stream);
int odc_scatter_accumulate_wide(const odc_layout_t *layout, const void *grad_full, void *const *accum64_shards,
                                void *stream);
int odc_retrieve_grads_wide(const odc_layout_t *layout, const void *const *accum64_shards, void *const *out_shards,
                            float scale, int out_dtype, void *stream);

/*
 * Hybrid sharding (Section 6.1, Appendix E).  Parameters and gradients are sharded only inside
 * a group of R devices (a node); the world is `groups` such groups, world rank w belongs to
 * group w / R with local rank w % R.  Every group holds a full copy of the parameter shards
 * and its own set of accumulator shards, so gather and scatter-accumulate never leave the
 * group; once per minibatch the groups' gradient shards are summed (the one step that crosses
 * nodes), and the optimizer states stay partitioned over all groups * R devices: device
 * (group k, owner r) keeps piece k of shard r, slots [k*P, (k+1)*P) with P = ceil(S_t / groups).
 *
 *   group-major arrays: [groups * R] host arrays of device pointers, entry k*R + r = group k's
 *   buffer of owner r (same sizes and alignment as in the plain calls).
 *
 * odc_hybrid_group_of            w / R, or -1 if w is outside [0, groups * R) or groups is bad.
 * odc_gather_hybrid              odc_gather from the shards of the worker's own group.
 * odc_scatter_accumulate_hybrid  odc_scatter_accumulate into the accumulators of the worker's own
 *                                group with its local rank; ordered mode and its history are per
 *                                group (ascending (local rank, microbatch) within a group).
 * odc_reduce_groups              minibatch end:
 *                                  out_shards[r][i] = ((a_0r[i] + a_1r[i]) + a_2r[i]) + ...  i valid
 *                                ascending group order, one binary32 add per further group (the
 *                                paper leaves the order open; this is the reading taken).
 *                                out_shards [R] may be group 0's accumulators (the sum replaces
 *                                them) but no other group's (ODC_ERR_INVALID_ARG).  Follow with
 *                                odc_retrieve_grads on out_shards.  Enqueues one kernel per 16
 *                                owners and per 8 groups.  (groups + 1) * 4 bytes per valid element.
 *                                The same call serves contributions that arrive concurrently on
 *                                one device without atomics: give every stream an accumulator
 *                                set of its own (ordered calls, one set per stream) and sum the
 *                                sets here; the result does not depend on how the streams
 *                                interleave.
 */
#define ODC_MAX_GROUPS 1024
int odc_hybrid_group_of(const odc_layout_t *layout, int groups, int world_worker);
int odc_gather_hybrid(const odc_layout_t *layout, int groups, const void *const *group_param_shards,
                      int world_worker, void *full_out, void *stream);
int odc_scatter_accumulate_hybrid(const odc_layout_t *layout, int groups, const void *grad_full,
                                  void *const *group_accum_shards, int world_worker, int microbatch,
                                  int flags, void *stream);
int odc_reduce_groups(const odc_layout_t *layout, int groups, const void *const *group_accum_shards,
                      void *const *out_shards, void *stream);

/*
 * Start of a minibatch (Section 3.2: accumulated gradients are retrieved at the minibatch
 * end, so accumulators are cleared before the next one): every valid accumulator element
 * becomes +0.0f.  Also clears the ordered-mode history of this accumulator set.
 * Algorithmic HBM traffic: 4 bytes per valid element.
 */
int odc_reset_accum(const odc_layout_t *layout, void *const *accum_shards, void *stream);

/*
 * Drop the ordered-mode history of an accumulator set without touching the accumulators (host
 * only, nothing enqueued): for accumulators that are about to be freed, or whose address has
 * just been handed out again.  Returns ODC_OK whether or not a history existed.
 */
int odc_forget_accum(const odc_layout_t *layout, void *const *accum_shards);

/* Text for an ODC_* code (static string, never NULL). */
const char *odc_strerror(int code);

/* hipError_t of the most recent failing HIP call on this host thread (0 if none). */
int odc_last_hip_error(void);

/*
 * Diagnostics, not part of the method.
 * odc_probe_copy: plain device-to-device copy kernel of `bytes` bytes (multiple of 16, both
 * pointers 16-byte aligned) on `stream`: a kernel of known traffic used to calibrate
 * hardware counters and to measure this GPU's copy ceiling next to the ODC kernels.
 * odc_tune: set a launch knob by name for all later calls of this process (safe to call while
 * other threads launch: every launch works from one consistent copy of the knobs):
 *   "gather_threads" / "accum_threads" / "reset_threads"  workgroup size of the single-tensor
 *                                                          kernels: 64, 128 or 256
 *   "gather_unroll" / "accum_unroll" / "reset_unroll"     16-byte work items per thread: 1, 2, 4
 *   "nontemporal"   0 or 1: streaming accesses carry the non-temporal hint
 *   "tile_remap"    0 or 1: each XCD sweeps its own contiguous eighth of the tiles
 *   "gather_store_sc1"  0 or 1: single-tensor gather stores carry sc1 + nt instead of nt
 *   "max_grid_x"    0 = one workgroup per tile; > 0 caps the grid, workgroups then loop
 *   "batch_rank_group"  owners handled by one workgroup of the multi-tensor accumulate,
 *                   retrieve and reset kernels: 0 = built-in choice (two for the
 *                   read-modify-write kernels when the launch is large enough, one for reset
 *                   and for small launches), or 1, 2, 4, 8
 *   "gather_tile_xcd_block"  multi-tensor gather: tiles are handed to the 8 XCDs in blocks of up to
 *                   this many consecutive tiles (a power of two up to 4096, default 16; 1 = plain
 *                   order; launches with few tiles take smaller blocks by themselves)
 *   "defaults"      with value 0: every knob back to its built-in default
 * Returns ODC_ERR_INVALID_ARG for an unknown name or a value out of range.  Results never
 * depend on the knobs.
 */
int odc_probe_copy(void *dst, const void *src, int64_t bytes, void *stream);
int odc_tune(const char *knob, int value);

#ifdef __cplusplus
}
#endif
#endif /* ODC_H */
