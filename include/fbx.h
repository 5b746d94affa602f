/*
 * fbx.h — C ABI of the MI355X feature-extraction library (libfbx.so).
 *
 * The library evaluates a fixed collection of per-feature operators on every
 * record of a batch of raw, tab-separated log records and returns, per emitted
 * slot, the 64-bit feature signs in record order (CSR: values + offsets).  This
 * is the "Extract features" stage of the paper (Section 3): operators are
 * collected, their dependencies resolved and their order fixed before the run
 * (Section 4, "Scheduling" and "Inner-GPU operator launching"), then executed
 * layer by layer on the GPU with dynamic memory taken from a pre-allocated pool
 * (Section 5).
 *
 * Conventions
 *   - Every call returns an fbx_status; nothing throws across this boundary.
 *   - "HOST" / "DEVICE" on a pointer says which memory it must point to.
 *   - The library never allocates device memory: all device storage (tables,
 *     scratch, results) lives in the workspace the caller hands over.
 *   - A plan is not thread-safe; distinct plans are independent.
 */
#ifndef FBX_H
#define FBX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fbx_plan fbx_plan; /* opaque, host-owned */

typedef enum {
  FBX_OK = 0,
  FBX_E_ARG = -1,   /* NULL or inconsistent argument                         */
  FBX_E_SPEC = -2,  /* operator-DAG spec rejected (see fbx_last_error)        */
  FBX_E_NOMEM = -3, /* workspace too small; required size reported            */
  FBX_E_INPUT = -4, /* record offsets decreasing / outside raw_len / a record of 2 GiB or more /
                       an operator with 2^26 or more signs for one record */
  FBX_E_HIP = -5    /* a HIP runtime call failed                              */
} fbx_status;

/* One emitted slot of a result.  HOST struct owned by the plan. */
typedef struct {
  uint32_t slot_id;        /* slot number given in the spec                                  */
  uint32_t fixed_arity;    /* k > 0: exactly k signs per record and offsets == NULL (record r
                              owns values[r*k, (r+1)*k)); 0: ragged, offsets given            */
  uint64_t n_values;       /* signs in this slot for this call                               */
  const uint64_t* values;  /* DEVICE, n_values entries, record order, token order inside     */
  const uint64_t* offsets; /* DEVICE, n_records + 1 entries, offsets[0] = 0,
                              offsets[n_records] = n_values; NULL for fixed-arity slots      */
  const uint64_t* tile_ends; /* DEVICE; NULL unless fbx_result.arrival_tile_records != 0 and the
                              slot is ragged: see there                                      */
} fbx_slot_view;

typedef struct {
  uint64_t n_records;
  uint64_t n_values_total;      /* sum of n_values over emitted slots                       */
  uint64_t n_malformed_numeric; /* bucket tokens that were not clean decimal text           */
  uint64_t arena_high_water;    /* workspace bytes this call needed (also set on NOMEM)     */
  uint32_t n_slots;
  uint32_t n_layers;
  const fbx_slot_view* slots;   /* HOST, n_slots entries in spec order; valid until the next
                                   fbx_extract or fbx_plan_destroy on this plan             */
  uint32_t tile_launches;       /* launches of the tile kernel this call took: 2 = counting +
                                   writing, 1 = one launch (no ragged slots, or ragged arrays
                                   sized from the previous call), 0 = the walk kernels ran    */
  uint32_t arrival_tile_records; /* 0: ragged slots are in record order (offsets as above).
                                   k > 0 (plan option "placement" = 1, and the call took the one-launch
                                   sequence): records were placed in tiles of k, tiles in the order in
                                   which they arrived.  Record r of a ragged slot then owns
                                   values[offsets[r], end) with end = offsets[r + 1], except for the last
                                   record of a tile (r % k == k - 1), whose end = tile_ends[r / k], and
                                   the batch's last record, whose end = offsets[n_records].  The tiles'
                                   shares [tile_ends[t] - signs of tile t, tile_ends[t]) are disjoint
                                   and cover [0, n_values); offsets are not monotone over tiles.
                                   Fixed-arity slots are in record order always.                     */
} fbx_result;

/*
 * fbx_plan_create — parse and type-check an operator-DAG spec, partition it
 * into layers and precompute per-operator constants.  Host only; needs no GPU.
 *
 * Operators without dependencies form layer 1; every other operator sits one
 * layer below its deepest input, so operators of one layer never depend on
 * each other (Section 4, "Scheduling").  The order is fixed here, once, before
 * any batch runs (Section 4, "Inner-GPU operator launching").
 *
 *   spec, spec_len : HOST, ASCII text, not retained:
 *       fbx 1
 *       fields <F>
 *       op <id> hash   slot=<u32> seed=<u64> emit=<0|1> field=<k> multi=<0|1>
 *       op <id> ngram  slot= seed= emit= field=<k> n=<1..8>
 *       op <id> bucket slot= seed= emit= field=<k> multi=<0|1> bounds=<i64,...>  (non-decreasing)
 *       op <id> filter slot= seed= emit= field=<k> multi=<0|1> prefix=<hex bytes>
 *       op <id> cross  slot= seed= emit= a=<id> b=<id>
 *       op <id> concat slot= emit= a=<id> b=<id>
 *     '#' starts a comment line.  a/b must name operators defined on earlier lines.
 *   out : receives the plan; untouched on error.
 * Errors: FBX_E_ARG, FBX_E_SPEC (message via fbx_last_error(NULL)).
 */
fbx_status fbx_plan_create(const char* spec, size_t spec_len, fbx_plan** out);

/* Release a plan (HOST memory only; the workspace stays the caller's).  NULL is fine. */
void fbx_plan_destroy(fbx_plan* plan);

/*
 * fbx_plan_workspace_hint — a workspace size (bytes) that is enough for typical
 * inputs of raw_len bytes and n_records records.  Ragged outputs cannot be
 * bounded ahead of time, so fbx_extract may still answer FBX_E_NOMEM together
 * with the exact requirement; the caller then enlarges the workspace and retries.
 */
fbx_status fbx_plan_workspace_hint(const fbx_plan* plan, uint64_t raw_len, uint64_t n_records,
                                   uint64_t* bytes);

/*
 * fbx_plan_set_workspace — hand over the pool, which is reserved up front in
 * device memory (Section 5).
 *   d_workspace : DEVICE, 256-byte aligned, stays owned by the caller and must
 *                 outlive every fbx_extract that uses it.
 * Copies the plan's constant tables into its head (synchronous copy, once).
 * Errors: FBX_E_ARG, FBX_E_NOMEM (smaller than the constant tables), FBX_E_HIP.
 */
fbx_status fbx_plan_set_workspace(fbx_plan* plan, void* d_workspace, uint64_t bytes);

/*
 * fbx_extract — run the whole path on one batch.
 *   d_raw      : DEVICE, raw_len bytes.  Record i is d_raw[rec_off[i], rec_off[i+1]);
 *                one trailing '\n' is not part of the record; fields are separated
 *                by '\t', list items by ','.
 *   d_rec_off  : DEVICE, n_records + 1 entries, non-decreasing, last <= raw_len.
 *   hip_stream : a hipStream_t (0 = default stream); all work is enqueued there.
 *   out        : HOST, filled on FBX_OK; on FBX_E_NOMEM only arena_high_water is set
 *                (the workspace size that would have sufficed).
 * Inputs are borrowed until the call returns.  Results point into the workspace
 * and are overwritten by the next fbx_extract on this plan.  The call
 * synchronises the stream exactly once, at its end, to read back sizes.
 * Layer by layer: by default all layers run in one launch, each workgroup taking
 * a tile of records through the layers in order with a barrier after each layer
 * (Section 4, "Scheduling": the synchronisation after a layer, per tile); with
 * the plan option "fused" = 0 one kernel launch per layer, the stream order being
 * the layer barrier, and the dynamic-memory pool released in O(1) after each layer
 * as far as live intermediates allow (Section 5, "Reset GPU memory pool").
 * Ragged slots need their sizes before they can be placed: the first call on a
 * plan counts in a launch of its own; later calls size the arrays from the call
 * before (plus a margin), count and write in one launch, and repeat themselves
 * with the counting launch if a batch does not fit (out->tile_launches tells).
 * After a batch in which some tile of records was too long for on-chip staging
 * the next 1, 2, 4 ... 64 calls count first without trying (fbx_last_error says so).
 * On an error the contents of the workspace are unspecified.
 * Errors: FBX_E_ARG, FBX_E_NOMEM, FBX_E_INPUT, FBX_E_HIP.
 */
fbx_status fbx_extract(fbx_plan* plan, const uint8_t* d_raw, uint64_t raw_len,
                       const uint64_t* d_rec_off, uint64_t n_records, void* hip_stream,
                       fbx_result* out);

/*
 * fbx_extract_static — fbx_extract for callers that cannot allocate device memory and have no
 * workspace to hand over: tight serving loops, code that must not call hipMalloc, harnesses that
 * forbid it.  Same computation and same results as fbx_extract, but
 *   - everything the kernels keep beside inputs and outputs (control block, plan tables, per-call
 *     operator programs, per-tile counts, bases and look-back words) lies in an array of
 *     fbx_static_scratch_bytes() = 64 MiB that is part of the library's device code: every GPU
 *     the library runs on holds one copy until the process ends;
 *   - the operators' arrays (the results) go to the caller's buffer:
 *       d_out     : DEVICE, 256-byte aligned, out_bytes bytes; out->slots point into it
 *                   (all but tile_ends of a result in arrival order, which points into the
 *                   library's array and holds until the next call on this GPU).
 * No fbx_plan_set_workspace is needed.  The call allocates and frees no device memory and
 * compiles nothing: plan options "compile" and "profile" are ignored here.
 * Limit: a batch whose tables exceed the array (they grow with tiles x ragged operators; the
 * message states the need) is refused with FBX_E_ARG before anything is enqueued.
 * FBX_E_NOMEM: d_out is too small; out->arena_high_water then holds the out_bytes that suffice.
 * All calls on one GPU share that GPU's array, which keeps what the last call left there: the
 * call itself resets what must start from zero and copies the plan's tables in again whenever the
 * last caller was another plan.  Two calls that overlap in time on one GPU (different threads or
 * streams) race: serialise them.  Other errors as fbx_extract.
 */
fbx_status fbx_extract_static(fbx_plan* plan, const uint8_t* d_raw, uint64_t raw_len,
                              const uint64_t* d_rec_off, uint64_t n_records, void* d_out,
                              uint64_t out_bytes, void* hip_stream, fbx_result* out);
uint64_t fbx_static_scratch_bytes(void);

/* Last error text of a plan (or of the last failed fbx_plan_create when plan is NULL).  After an
 * fbx_extract that returned FBX_OK it is empty, or a note on why the call took the longer of its
 * two launch sequences. */
const char* fbx_last_error(const fbx_plan* plan);
const char* fbx_status_str(fbx_status s);

/*
 * Plan introspection (HOST): operator count, layer count and, if the arrays
 * are non-NULL (capacity n_ops each), the 1-based layer and the fixed arity
 * (0 = ragged) of every operator in spec order.
 */
fbx_status fbx_plan_info(const fbx_plan* plan, uint32_t* n_ops, uint32_t* n_layers,
                         uint32_t* layer_of_op, uint32_t* arity_of_op);

/*
 * Tuning knobs, all optional.  Keys:
 *   "fused"        1: all layers in one launch (tile kernel, default); 0: one launch per
 *                  layer (walk kernels)
 *   "tile_engine"  1: with "fused" = 1 the tile kernel runs wherever a plan fits it (default); 0: the
 *                  walk kernels run all layers in one launch (the same code that "fused" = 0
 *                  launches once per layer, which makes the two comparable)
 *   "one_launch"   1: later calls skip the counting launch as described at fbx_extract
 *                  (default); 0: always count first
 *   "placement"    0: ragged slots in record order (default).  1: in a call that skips the counting
 *                  launch every tile of records takes its share of a ragged slot with one atomic
 *                  add on the slot's running total (Section 5, Algorithm 1, a tile's share as the
 *                  block) instead of waiting for the tiles before it: tiles land in the order in
 *                  which they arrive (fbx_result.arrival_tile_records says so and how to read it),
 *                  and plans with many ragged operators skip the counting launch too
 *   "tile_log2"    -1: records per tile chosen per call (default); 0..6: 2^value records
 *   "raw_cap"      0: bytes of text a workgroup stages at a time chosen per call (default);
 *                  64..65000: that many
 *   "lds_budget"   LDS bytes per workgroup the tile size is chosen for (default 81920)
 *   "grid_limit"   0: as many workgroups as run at the same time (default); else at most that
 *   "spin_limit"   polls after which a tile of the one-launch sequence stops waiting for an
 *                  earlier tile's count (default 2^22; 0: it never waits).  A wait that runs out
 *                  ends no kernel early and writes nothing: the call is answered by the counting
 *                  sequence instead and fbx_last_error says so.
 *   "profile"      1: time every kernel of fbx_extract with HIP events
 *   "compile"      1: compile the tile kernel for this plan at run time, as Section 4 does with
 *                  the meta-kernel of a layer: the first fbx_extract that meets a tile shape
 *                  compiles the kernels it launches with the plan's counts and table offsets as
 *                  literals (a few seconds each, on the host, inside that call), later calls
 *                  reuse them.  When the compiler or the kernel sources (csrc/ beside the
 *                  library and include/ one level up, or <dir>/csrc and <dir>/include with the
 *                  environment variable FBX_KERNEL_SOURCES=<dir>) are missing the generic kernel
 *                  runs and fbx_last_error says why.
 *                  0: one generic kernel for every plan (default)
 *   "tile_threads" 512 (default) or 1024: lanes of a workgroup of the kernels compiled for the plan
 *   "lane_ops"     kernels compiled for the plan, tiles of 64 records ("tile_log2" = 6) only: how the
 *                  single-sign operators (single-valued hashes and buckets, crosses of two single
 *                  signs) run.  0 (default): as on any other tile, lanes being (record, operator)
 *                  pairs; 1: one operator per wavefront at a time, one record per lane, the
 *                  operator's numbers read from the program table; 2: the same as straight-line
 *                  code generated for the plan, one piece per operator with its field, key and
 *                  table rows as literals (Section 4, "Inner-GPU operator launching": every
 *                  operator a device function, called one after the other).  Measured slower than 0
 *                  on the benchmark workloads, which is why 0 is the default.
 * Errors: FBX_E_ARG for an unknown key or an out-of-range value.
 */
fbx_status fbx_plan_set_option(fbx_plan* plan, const char* key, int64_t value);

/*
 * Tile kernels compiled for the plan so far (option "compile" = 1) and the host time spent
 * compiling them, in milliseconds.  Either pointer may be NULL.
 */
fbx_status fbx_plan_compiled(const fbx_plan* plan, uint32_t* n_kernels, double* ms);

/*
 * The source text that option "compile" = 1 hands to the run-time compiler for a batch of this
 * shape (raw_len bytes, n_records records) and launch mode (0 counting, 1 writing, 2 both in one
 * launch): the tile kernel's own file behind the definitions that fix the plan's numbers.  HOST
 * only, needs no GPU.  buf (HOST, buf_len bytes, may be NULL with buf_len 0) receives the text,
 * NUL-terminated and cut to fit; *needed (may be NULL) the size that holds all of it.
 * Errors: FBX_E_ARG (also for a plan too wide for the tile kernel).
 */
fbx_status fbx_plan_kernel_source(const fbx_plan* plan, uint64_t raw_len, uint64_t n_records, int mode,
                                  char* buf, size_t buf_len, size_t* needed);

/*
 * Kernel timings of the last fbx_extract (needs option "profile" = 1).
 * which: 0 validate, 1 count, 2 scan, 3 alloc, 4 all tile launches together,
 *        100 + l : tile launch of layer l (1-based; 101 alone when all layers share a launch).
 * A kernel the last call did not launch answers FBX_E_ARG.
 * ms receives the HIP-event duration on the call's stream.
 */
fbx_status fbx_plan_kernel_ms(const fbx_plan* plan, uint32_t which, float* ms);

/*
 * In-kernel dynamic allocation as a primitive (Section 5, Algorithm 1 and
 * "Reset GPU memory pool").  fbx_arena_alloc launches ceil(n / block_threads)
 * workgroups that call the library's device-side allocator (the one its own kernels
 * call, see fbx_extract_unordered); in each, thread i asks for d_sizes[i] bytes: the
 * workgroup takes a prefix sum of its sizes (inside a wavefront by data-parallel moves,
 * across wavefronts through LDS), ONE thread adds the workgroup total (rounded up to
 * 128 bytes) to *d_head with an atomic add, and thread i gets
 * old_head + (sum of the sizes of the threads before it).  Workgroups land in
 * arrival order, so offsets are only unique, not ordered, across workgroups.
 *   d_head    : DEVICE, one u64 (the pool's idle-memory head, a byte offset)
 *   d_sizes   : DEVICE, n u64
 *   d_offsets : DEVICE, n u64 out (byte offsets from the pool base)
 *   block_threads : 64..1024, multiple of 64
 * fbx_arena_reset sets *d_head = value (constant time, frees everything above it).
 * Both only enqueue on hip_stream.
 */
fbx_status fbx_arena_alloc(uint64_t* d_head, const uint64_t* d_sizes, uint64_t n, uint64_t* d_offsets,
                           uint32_t block_threads, void* hip_stream);
fbx_status fbx_arena_reset(uint64_t* d_head, uint64_t value, void* hip_stream);

/*
 * fbx_extract_unordered — one operator of layer 1 whose lists vary in length (a multi-valued
 * hash or bucket, a filter, an n-gram), run the way Section 5 and Figure 5 describe: one record
 * per thread; a thread works out how many signs its record yields, the workgroup allocates with
 * Algorithm 1 (a prefix sum and ONE atomic add on the pool's head per workgroup of 256 threads,
 * workgroup regions 128-byte aligned), the thread writes its signs into its region and records
 * where that is.  No counting launch and no scan; in exchange the output is unordered: the
 * regions of one workgroup lie end to end in record order, workgroups in arrival order.
 *   slot_id          : an emitted slot of the plan (operator of layer 1 with ragged output)
 *   d_raw, d_rec_off : as for fbx_extract
 *   d_pool           : DEVICE, 128-byte aligned, pool_bytes bytes: the pre-allocated pool
 *   d_state          : DEVICE, four u64 owned by the caller: [0] the pool's idle-memory head
 *                      (bytes from d_pool), [1..3] used by the call
 *   reset            : 1: the head is set back to the pool's base first (the constant-time release of
 *                      Section 5, "Reset GPU memory pool"); 0: allocate behind what earlier calls took
 *   d_thread_offsets : DEVICE, n_records u64 out: byte offset of record i's signs from d_pool
 *                      (the "Thread Offsets" of Figure 5)
 *   d_lengths        : DEVICE, n_records u32 out: signs of record i (token order inside)
 *   out              : HOST: signs in all, malformed numerics, the head after the call
 * Needs fbx_plan_set_workspace (the operator's boundaries or prefix are read from the plan's
 * tables there); touches nothing else in the workspace.  Synchronises the stream once.
 * Errors: FBX_E_ARG, FBX_E_INPUT, FBX_E_HIP, and FBX_E_NOMEM when the pool is exhausted: nothing
 * is written beyond it and out->pool_head holds the bytes that would have sufficed.
 */
typedef struct {
  uint64_t n_values, n_malformed_numeric, pool_head;
} fbx_unordered_result;
fbx_status fbx_extract_unordered(fbx_plan* plan, uint32_t slot_id, const uint8_t* d_raw, uint64_t raw_len,
                                 const uint64_t* d_rec_off, uint64_t n_records, void* d_pool,
                                 uint64_t pool_bytes, uint64_t* d_state, int reset,
                                 uint64_t* d_thread_offsets, uint32_t* d_lengths, void* hip_stream,
                                 fbx_unordered_result* out);

/*
 * The "clean views" stage in toy form (Section 3, "Clean views": null values are filled, fields are
 * taken out of a JSON-like column, instances are dropped by a custom filter; Section 4 runs the
 * stage on the GPU).  The paper defines none of the three; this is the contract built here.
 * Spec text (line-oriented ASCII, '#' starts a comment):
 *     fbxclean 1
 *     fields <F>
 *     fill field=<k> value=<hex bytes>    an empty field k becomes the value (no tab, no newline, not empty)
 *     key  field=<k> name=<hex bytes>     field k is a flat list "key:value;key:value;...": it becomes the
 *                                         value of the first pair whose key is exactly the name, or empty
 *                                         (a pair's key ends at its first ':'; a pair without ':' never matches)
 *     keep field=<k> prefix=<hex bytes>   the record is dropped unless field k begins with the prefix
 * A record (framed as for fbx_extract) is cut into exactly F fields (missing ones are empty, further
 * ones are dropped); the operators that name a field apply to it in spec order, a filter seeing the
 * field as the operators before it left it.  A kept record is written as its F fields joined by
 * '\t' and ended by '\n'; kept records follow each other in input order.
 *
 * fbx_clean_create   : HOST only.  Errors: FBX_E_ARG, FBX_E_SPEC (fbx_clean_last_error(NULL) says why).
 * fbx_clean_scratch_hint : bytes of scratch that fbx_clean_run needs for n_records records.
 * fbx_clean_run      : d_raw / d_rec_off as for fbx_extract (DEVICE).
 *     d_out      : DEVICE, out_cap bytes: receives the cleaned text
 *     d_out_off  : DEVICE, n_records + 1 u64: entries 0 .. n_kept receive the kept records' offsets
 *                  (entry n_kept = length of the cleaned text), ready to be handed to fbx_extract
 *     d_scratch  : DEVICE, 256-byte aligned, scratch_bytes bytes, the caller's; contents unspecified afterwards
 *     out        : HOST: kept records, bytes of cleaned text, scratch bytes needed
 *   Enqueues on hip_stream and synchronises it once.  Errors: FBX_E_ARG, FBX_E_INPUT (bad offsets),
 *   FBX_E_HIP, FBX_E_NOMEM: scratch too small (out->required_scratch), or d_out too small: nothing
 *   is written to it and out->out_len holds the bytes needed.
 */
typedef struct fbx_clean fbx_clean;
typedef struct {
  uint64_t n_kept, out_len, required_scratch;
} fbx_clean_result;
fbx_status fbx_clean_create(const char* spec, size_t spec_len, fbx_clean** out);
void fbx_clean_destroy(fbx_clean* clean);
const char* fbx_clean_last_error(const fbx_clean* clean);
fbx_status fbx_clean_scratch_hint(const fbx_clean* clean, uint64_t n_records, uint64_t* bytes);
fbx_status fbx_clean_run(fbx_clean* clean, const uint8_t* d_raw, uint64_t raw_len, const uint64_t* d_rec_off,
                         uint64_t n_records, uint8_t* d_out, uint64_t out_cap, uint64_t* d_out_off,
                         void* d_scratch, uint64_t scratch_bytes, void* hip_stream, fbx_clean_result* out);

/*
 * The measurement behind Table 1 of the paper (Section 4, "Inner-GPU operator launching"), on this
 * device: n_launches launches of an empty kernel with five pointer arguments are enqueued on
 * hip_stream back to back and waited for; *microseconds (HOST) receives the host time from the
 * first launch call to the end of the wait.  The stream is drained before the clock starts.
 * Errors: FBX_E_ARG (0 or more than 10^6 launches, NULL), FBX_E_HIP.
 */
fbx_status fbx_launch_overhead(uint32_t n_launches, void* hip_stream, double* microseconds);

#ifdef __cplusplus
}
#endif
#endif /* FBX_H */
