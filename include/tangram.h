/*
 * tangram.h -- C ABI of the Reuse Store's Load path on one MI355X.
 *
 * The library implements, for one GPU, what the paper's Section 3.1 asks of a
 * worker's Reuse Store when a model is switched in: look every tensor of the
 * model up in the Tensor Mapping (indexed by a per-tensor fingerprint),
 * allocate pool space for what must be placed (Section 3.2: Region List,
 * best-fit), bring in the missing tensors from the CPU-side Model Cache,
 * update the mapping, and hand back the GPU address of every tensor.
 *
 * Conventions that hold for every entry point
 *  - Pointers marked [host] are ordinary host pointers read or written by the
 *    CPU during the call.  Pointers marked [device] are HIP device addresses
 *    and are only ever dereferenced by kernels or the copy engine.  Pointers
 *    marked [pinned host] must be page-locked memory obtained from
 *    hipHostMalloc (torch's pin_memory=True): the copy engine reads it, and
 *    kernels read it through its device mapping.
 *  - Ownership: the caller owns the pool slab, every host buffer and every
 *    stream, and keeps them alive while the library uses them.  The library
 *    owns its metadata and a small amount of device / pinned scratch
 *    (descriptor tables, result words, events).  Every pool has scratch of
 *    its own, allocated on first use and freed by tg_pool_destroy; the calls
 *    that take no pool (tg_fingerprint, tg_compare) share one more, kept
 *    until tg_shutdown() or process exit.
 *  - Streams are hipStream_t values passed as void* (NULL = the null stream).
 *  - Errors: every function returns a tg_status; 0 is success, negative
 *    values are errors, out-parameters are left untouched on error, and no
 *    call aborts or throws across the boundary.  A failed tg_plan leaves
 *    the pool's metadata exactly as it was; so does a failed tg_assemble,
 *    except where its comment says otherwise (a plan that had already moved
 *    or overwritten resident tensors when it failed).
 *  - Threading: a pool is externally synchronised (one caller at a time per
 *    pool); different pools share nothing, so they may be used from different
 *    threads at the same time, loads included.  tg_fingerprint / tg_compare
 *    may be called from several threads; they serialise on their scratch.
 *    There is no process-wide setting: launch shape and profiling belong to a
 *    pool, timings to a plan.
 *  - Device: a pool's scratch lives on the GPU that is current at the pool's
 *    first call that touches the device (likewise for the calls that take no
 *    pool); calls made with another device current return TG_ERR_INVALID.
 *  - All sizes and offsets are in bytes.  Integer arithmetic of the
 *    fingerprint is unsigned 64-bit and wraps.
 */
#ifndef TANGRAM_H
#define TANGRAM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t tg_status;

#define TG_OK             0
#define TG_ERR_INVALID   (-1)  /* null pointer, zero length, overflow, misalignment, duplicate active model */
#define TG_ERR_NOSPACE   (-2)  /* no placement for every tensor of the model */
#define TG_ERR_STALE     (-3)  /* the pool changed between tg_plan and tg_assemble */
#define TG_ERR_NOTFOUND  (-4)  /* unknown model id */
#define TG_ERR_HIP       (-5)  /* a HIP call failed (no device, launch or copy error) */
#define TG_ERR_NOMEM     (-6)  /* host or scratch allocation failed */
#define TG_ERR_CORRUPT   (-7)  /* TG_ASSEMBLE_VERIFY: an assembled tensor's fingerprint differs from its descriptor */

/* tg_plan flags */
#define TG_PLAN_CONFIRM   1u   /* compare bytes of every fingerprint hit before trusting it */
#define TG_PLAN_EVICT     2u   /* Stage 1: evict retained tensors by ascending cost when free bytes are short */
#define TG_PLAN_MERGE     4u   /* Stage 2: when best fit fails, pack by partitions and merge free regions */
#define TG_PLAN_ALIAS     8u   /* a hit is used where it lies (no copy, no new slot) */
#define TG_PLAN_PACK_TEXT 16u  /* Stage 2 packing test as the text words it (see tg_plan) */
#define TG_PLAN_CAP_TEXT  32u  /* Stage 2 subspace capacity as the text defines it (see tg_plan) */
/* tg_assemble flags */
#define TG_ASSEMBLE_VERIFY 1u  /* fingerprint every assembled slot and compare with the descriptor */
/* tg_release flags */
#define TG_RELEASE_EVICT  1u   /* free the model's regions now instead of retaining them */

/* tg_plan_op.kind */
#define TG_OP_REUSE 0u         /* device-to-device copy from a resident tensor */
#define TG_OP_H2D   1u         /* transfer from the model's pinned host buffer */

typedef struct tg_pool tg_pool;            /* opaque; library-owned metadata of one Unified Memory Pool */
typedef struct tg_load_plan tg_load_plan;  /* opaque; freed by tg_plan_free */

/* A byte extent to fingerprint.  ptr [device] must be 16-byte aligned. */
typedef struct {
    const void *ptr;
    uint64_t    nbytes;
} tg_span;

/* Two extents to compare.  a, b [device] must be 16-byte aligned. */
typedef struct {
    const void *a;
    const void *b;
    uint64_t    nbytes;
} tg_pair;

/* One tensor of an incoming model: its length, its fingerprint (from
 * tg_fingerprint at registration) and where its bytes start inside the
 * model's host buffer. */
typedef struct {
    uint64_t nbytes;
    uint64_t fp;
    uint64_t src_off;
} tg_tensor_desc;

/* An incoming model.  host_base [pinned host] .. host_base + host_bytes is
 * the model's image in the Model Cache; tensors [host] has n_tensors rows in
 * the model's canonical tensor order.  host_base may be NULL (host_bytes 0)
 * for a model whose bytes are not all in pinned memory at once: planning
 * needs only (nbytes, fp) per tensor, src_off is then the caller's own
 * reference (it is echoed in the plan's rows), and the missing tensors are
 * handed over piece by piece with tg_assemble_begin / _feed / _wait. */
typedef struct {
    uint64_t              model_id;
    const void           *host_base;
    uint64_t              host_bytes;
    uint32_t              n_tensors;
    uint32_t              reserved;   /* must be 0 */
    const tg_tensor_desc *tensors;
} tg_model_desc;

/* What will happen to tensor k of the planned model.
 * kind == TG_OP_REUSE: pool[dst_off .. +nbytes) = pool[src_off .. +nbytes)
 * kind == TG_OP_H2D  : pool[dst_off .. +nbytes) = host_base[src_off .. +nbytes) */
typedef struct {
    uint32_t kind;
    uint32_t reserved;
    uint64_t dst_off;
    uint64_t src_off;
    uint64_t nbytes;
} tg_plan_op;

/* A resident tensor that Stage 2 moves to merge free regions. */
typedef struct {
    uint64_t old_off;
    uint64_t new_off;
    uint64_t nbytes;
} tg_move;

/* Totals of a plan. */
typedef struct {
    uint32_t n_tensors;
    uint32_t n_evictions;     /* tensors Stage 1 evicts */
    uint32_t n_moves;         /* tensors Stage 2 moves */
    uint32_t alias;           /* 1 if the plan was made with TG_PLAN_ALIAS */
    uint32_t n_reused;        /* tensors found resident (rows of kind TG_OP_REUSE) */
    uint32_t reserved;
    uint64_t reused_bytes;    /* bytes found resident */
    uint64_t transfer_bytes;  /* bytes that come from the host */
    uint64_t copy_bytes;      /* bytes the gather kernel copies (0 in alias mode) */
    uint64_t evicted_bytes;   /* slot bytes Stage 1 frees */
    uint64_t moved_bytes;     /* bytes of the tensors Stage 2 moves */
    uint64_t merge_bound;     /* Algorithm 1's merge cost M (an upper bound on moved slot bytes) */
} tg_plan_summary;

typedef struct {
    uint64_t capacity;        /* pool size */
    uint64_t free_bytes;      /* sum of free regions */
    uint64_t largest_free;    /* longest free region */
    uint64_t n_regions;       /* Region List length (free + allocated) */
    uint64_t n_free_regions;
    uint64_t n_entries;       /* Tensor Mapping rows (active + inactive) */
    uint64_t n_active;        /* rows that belong to an active model */
    uint64_t generation;      /* bumped by every commit and release */
} tg_stats;

/* Durations, in milliseconds, of the device work one plan caused, measured
 * with HIP events on the stream the work ran on (tg_plan_timing).  The device
 * fields are filled only if the pool had profiling on (tg_pool_set_profiling)
 * when the plan was made and carried out; a field is 0 if that work did not
 * run. */
typedef struct {
    float    compare_ms;      /* compare kernel of a confirming tg_plan */
    float    gather_ms;       /* the gather kernel */
    float    h2d_ms;          /* first to last host-to-device copy, summed over the feeds */
    float    verify_ms;       /* fingerprint kernels of a verifying assemble, summed */
    float    plan_host_ms;    /* host time of tg_plan (steady clock; always filled) */
    float    move_ms;         /* first to last merge-move launch */
    uint64_t compare_bytes, gather_bytes, h2d_bytes, verify_bytes;
    uint32_t h2d_copies;      /* hipMemcpyAsync calls issued */
    uint32_t move_launches;   /* copy launches the merge moves took */
    uint32_t verify_launches; /* fingerprint launches of a verifying assemble (verify_ms is their sum) */
    uint32_t feeds;           /* tg_assemble_feed calls (1 for a load from a whole host image) */
    uint64_t move_bytes;      /* bytes of the tensors moved */
    uint64_t move_traffic_bytes; /* bytes read + written by the move launches (staged stretches count twice) */
    uint64_t fused_verify_bytes; /* bytes a verifying load fingerprinted inside its copy launches (not in verify_bytes) */
} tg_timing;

/*
 * Pool.  (Section 3.1: one Unified Memory Pool per GPU; Section 3.2: the pool
 * is a Region List of free / allocated regions in physical order.)
 *
 * dev_base [device] is the slab, capacity its length; both must be multiples
 * of align, and align a power of two >= 16 (256 is the usual choice).  The
 * library never allocates, frees or touches the slab here; it records the
 * base so that offsets can be turned into addresses.  *out receives the pool.
 * TG_ERR_INVALID on null / zero / misaligned arguments.
 */
tg_status tg_pool_create(void *dev_base, uint64_t capacity, uint32_t align, tg_pool **out);

/* Frees the pool's metadata.  The slab is not touched.  NULL is accepted. */
tg_status tg_pool_destroy(tg_pool *pool);

/* Snapshot of the pool's counters.  out [host]. */
tg_status tg_pool_stats(const tg_pool *pool, tg_stats *out);

/* One region of the Region List (Section 3.2): [off, off + len) is free or
 * holds one tensor's slot. */
typedef struct {
    uint64_t off;
    uint64_t len;
    uint32_t free;            /* 1 free, 0 allocated */
    uint32_t reserved;
} tg_region;

/* One row of the Tensor Mapping (Section 3.1): a resident tensor. */
typedef struct {
    uint64_t off;             /* slot offset in the pool */
    uint64_t nbytes;
    uint64_t fp;
    uint32_t n_owners;        /* models that list it (retained or running) */
    uint32_t active_refs;     /* running models that use it; 0 = evictable */
} tg_entry;

/*
 * The Region List in physical order, and the Tensor Mapping in ascending
 * pool offset.  out [host] has room for cap rows; *n receives the number of
 * rows the pool holds, and min(*n, cap) rows are written (call with cap 0 to
 * size the array).  For inspection and tests; a load never needs them.
 */
tg_status tg_pool_regions(const tg_pool *pool, tg_region *out, uint32_t cap, uint32_t *n);
tg_status tg_pool_entries(const tg_pool *pool, tg_entry *out, uint32_t cap, uint32_t *n);

/*
 * Launch shape of the three streaming kernels, and two thresholds of the
 * host-to-device stream.  *_unroll is the number of independent 128-bit loads
 * a lane issues per tile (2, 4, 8 or 16; a tile is lanes x 16 B x unroll, with
 * 256 lanes for fingerprint and compare and 1024 for the gather);
 * *_wgs_per_cu is the number of workgroups launched per compute unit.
 * h2d_kernel_max_bytes > 0 lets missing tensors up to that size be fetched by
 * the gather kernel through the pinned buffer's device mapping instead of one
 * copy-engine call each (default 64 KiB: such a copy takes about 1 us on the
 * link and about 10 us to issue).  h2d_group_bytes is the copy-grouping
 * threshold of Section 4: missing tensors that are adjacent both in the host
 * image and in the pool are merged into one copy until the copy exceeds this
 * many bytes (the paper's loader uses 8 MB); 0, the default, puts no limit on
 * a merged copy.  fuse_verify is a pair of bits.  Bit 0 (set by default) makes
 * a verifying load compute the fingerprints of the tensors it copies device to
 * device inside the gather launch, from the bytes as they pass through the
 * registers, instead of reading the written slots again with a second launch:
 * one pass over HBM less, and it vouches for what was read rather than for
 * what was written.  Bit 1 (clear by default) does the same for the tensors a
 * merge moves (one that is cut into pieces, or staged, is summed piece by piece
 * by the launches that write it to its new place); by default they are
 * fingerprinted where they landed by a launch of their own, which runs beside
 * the host-to-device copies, whereas the move launches hold those copies up.
 * The defaults (tg_default_tuning) are the measured optimum on
 * MI355X; results never depend on these values.  A pool starts with the
 * defaults.
 */
typedef struct {
    uint32_t fingerprint_unroll, fingerprint_wgs_per_cu;
    uint32_t gather_unroll, gather_wgs_per_cu;
    uint32_t compare_unroll, compare_wgs_per_cu;
    uint64_t h2d_kernel_max_bytes;
    uint64_t h2d_group_bytes;
    uint32_t fuse_verify;     /* bit 0: a verifying load fingerprints copied tensors inside the copy launch; bit 1: moved tensors too */
    uint32_t reserved;        /* must be 0 */
} tg_tuning;
tg_status tg_default_tuning(tg_tuning *out);
tg_status tg_pool_set_tuning(tg_pool *pool, const tg_tuning *t);
tg_status tg_pool_get_tuning(const tg_pool *pool, tg_tuning *out);

/*
 * Profiling switch of a pool: while it is on, the plans made for the pool
 * record HIP events around their device work (see tg_timing, tg_plan_timing).
 * Off by default; recording costs a few microseconds per launch.
 */
tg_status tg_pool_set_profiling(tg_pool *pool, int on);

/*
 * Measurement aid: words per second that this GPU's integer units sustain on
 * the fingerprint's arithmetic alone -- one launch in which every lane mixes
 * iters x 16 words made up in registers, no memory traffic -- timed with HIP
 * events on `stream`.  Times eight bytes it is the bandwidth above which the
 * fingerprint kernel would be bound by arithmetic rather than by HBM.
 * TG_ERR_INVALID unless 1 <= iters <= 2^20.
 */
tg_status tg_measure_mix_rate(uint32_t iters, void *stream, double *words_per_s);

/*
 * Fingerprint.  (Section 3.1: every tensor has a fingerprint that indexes the
 * Tensor Mapping.  The function: with gamma = 0x9E3779B97F4A7C15 and
 * SM(x) = SplitMix64's output for the not-yet-advanced state x,
 *     F = sum over i of SM(w_i XOR i*gamma)   (mod 2^64)
 * over the little-endian 64-bit words w_i of the extent, i from 0, bytes past
 * the end reading as zero; the empty extent has F = 0.)
 *
 * spans [host] has n rows whose ptr fields are [device] addresses (pinned
 * host memory may be passed by its device mapping).  One kernel launch on
 * `stream` covers all spans; the call waits for it and writes out_fp[0..n)
 * [host].  n == 0 succeeds and does nothing.  TG_ERR_INVALID for a null
 * array, a null ptr with nbytes > 0, or a ptr that is not 16-byte aligned.
 */
tg_status tg_fingerprint(const tg_span *spans, uint32_t n, uint64_t *out_fp, void *stream);

/* tg_fingerprint with a launch shape of the caller's (tuning; NULL = the
 * defaults) and, if kernel_ms [host] is not NULL, the kernel's duration in
 * milliseconds measured with HIP events on `stream` (0 when no byte was read). */
tg_status tg_fingerprint_ex(const tg_span *spans, uint32_t n, uint64_t *out_fp, void *stream,
                            const tg_tuning *tuning, float *kernel_ms);

/*
 * tg_fingerprint for callers that cannot allocate: code that runs where
 * hipMalloc is forbidden or too slow (a tight serving loop that re-checks
 * resident tensors, a harness that forbids allocation, code around a HIP
 * graph capture).  Same arguments, same results, same errors as
 * tg_fingerprint, with these differences:
 *  - the span table, the tile table and the result words live in a fixed
 *    128 KiB array that is part of the library's code object (one copy per
 *    GPU, held from the moment the library is loaded on that GPU until the
 *    process ends); the call makes no hipMalloc, hipFree or hipHostMalloc, creates
 *    no events and allocates no host memory;
 *  - n may be at most TG_NOALLOC_MAX_SPANS; more is TG_ERR_INVALID;
 *  - it works on whichever GPU is current (the array's address is looked up
 *    once per GPU, at the first call made with that GPU current), and always
 *    with the default launch shape.
 * Every call on a GPU uses that GPU's one array, which keeps the previous
 * call's contents; the call clears the words it adds into.  Calls from one
 * process are serialised by the library and each waits for its kernel, so they
 * cannot overlap; two processes have separate copies.
 */
#define TG_NOALLOC_MAX_SPANS 4096u
tg_status tg_fingerprint_noalloc(const tg_span *spans, uint32_t n, uint64_t *out_fp, void *stream);

/*
 * Bytewise comparison of n pairs of extents in one launch on `stream`;
 * out_differs[i] [host] is 0 when pair i holds identical bytes and 1
 * otherwise.  (The confirmation step behind a fingerprint hit; the paper
 * treats fingerprints as unique, Section 3.1.)  The call waits for the kernel.
 */
tg_status tg_compare(const tg_pair *pairs, uint32_t n, uint32_t *out_differs, void *stream);

/* tg_compare with a launch shape of the caller's and the kernel's duration,
 * as tg_fingerprint_ex. */
tg_status tg_compare_ex(const tg_pair *pairs, uint32_t n, uint32_t *out_differs, void *stream,
                        const tg_tuning *tuning, float *kernel_ms);

/*
 * Plan the load of `model` into `pool`.  (Section 3.1: search the Tensor
 * Mapping for the model's tensors, evict tensors of inactive models if space
 * is short; Section 3.2: best-fit allocation, Stage 1 minimal-cost eviction,
 * Stage 2 Partitioned-Gain Packing.)
 *
 *  match    key (fp, nbytes) against the tensors resident when the call
 *           starts (in use or retained); among equal keys the lowest pool
 *           offset wins.  With TG_PLAN_CONFIRM every candidate is compared
 *           with the incoming bytes (read from host_base through its device
 *           mapping by the compare kernel on `stream`) and candidates whose
 *           bytes differ are dropped.  A tensor with a surviving candidate is
 *           a TG_OP_REUSE, any other a TG_OP_H2D.
 *  slots    by default every tensor gets a fresh slot of roundup(nbytes,
 *           align) bytes and a hit is copied into it.  With TG_PLAN_ALIAS a
 *           hit is used where it lies (dst_off == src_off, the row becomes
 *           shared between the models that own it) and only misses get slots.
 *  evict    with TG_PLAN_EVICT, when the free bytes are fewer than the slots
 *           need: tensors that no running model uses and that this plan does
 *           not read are evicted in ascending cost c = p * (nbytes / b) * alpha
 *           of their model (Eq. 2; see tg_set_model_cost; a tensor several
 *           models own costs the sum; ties: lower offset) until enough bytes
 *           are free.
 *  allocate largest slot first (ties: lower index first), each into the
 *           smallest free region that holds it (ties: lowest offset), at the
 *           region's low end.
 *  merge    with TG_PLAN_MERGE, when best fit fails although enough bytes are
 *           free: Algorithm 1 cuts the Region List at resident tensors
 *           (largest first) wherever its two-bin packing test lets the new
 *           tensors be divided over the two sides; each final subspace that
 *           was given tensors takes them by best fit if it can, else its
 *           resident tensors are slid to its low end (tg_plan_moves) and the
 *           tensors placed in the merged free tail.  merge_bound is the sum of
 *           the resident bytes inside those subspaces.  Tensors in use by a
 *           running model never move: they cut the pool into subspaces
 *           beforehand, and each new tensor (largest first) goes to the one
 *           with the most room left.  Two points where the paper's text and
 *           its listing part ways are selectable.  The packing test is the
 *           listing's (a tensor must be smaller than the smaller bin's
 *           remaining room; it goes to the bin with more room); the text
 *           lets the tensor merely fit the bin with more room, which
 *           TG_PLAN_PACK_TEXT selects and which splits far more often.  A
 *           subspace's room is its free bytes; the text defines its capacity
 *           as free plus allocated bytes, which TG_PLAN_CAP_TEXT selects and
 *           which can hand a subspace more than it can hold after merging --
 *           the plan then fails with TG_ERR_NOSPACE.
 *
 * The pool is not modified.  *out receives a plan bound to the pool's current
 * generation.  TG_ERR_INVALID: null arguments, unknown flag bits, n_tensors ==
 * 0, a zero-length tensor, src_off + nbytes > host_bytes (when the model has
 * a host image), TG_PLAN_CONFIRM without a host image, model_id running in
 * the pool.  TG_ERR_NOSPACE: the tensors cannot be placed with the stages
 * that the flags allow.  `stream` is used only with TG_PLAN_CONFIRM.
 */
tg_status tg_plan(tg_pool *pool, const tg_model_desc *model, uint32_t flags, void *stream,
                  tg_load_plan **out);

/* Rows of the plan, one per tensor in the model's order, and byte totals:
 * reused_bytes + transfer_bytes == sum of nbytes.  A REUSE row's src_off is
 * where the resident copy lies once the plan's moves have run.  *ops points
 * into the plan and lives until tg_plan_free.  Any out pointer may be NULL. */
tg_status tg_plan_ops(const tg_load_plan *plan, const tg_plan_op **ops, uint32_t *n,
                      uint64_t *reused_bytes, uint64_t *transfer_bytes);

/* Totals of the plan.  out [host]. */
tg_status tg_plan_info(const tg_load_plan *plan, tg_plan_summary *out);

/* The tensors Stage 2 moves, in the order the moves are carried out, and the
 * pool offsets of the tensors Stage 1 evicts, in eviction order.  The arrays
 * live in the plan until tg_plan_free. */
tg_status tg_plan_moves(const tg_load_plan *plan, const tg_move **moves, uint32_t *n);
tg_status tg_plan_evictions(const tg_load_plan *plan, const uint64_t **offsets, uint32_t *n);

/* What the plan's device work took (see tg_timing); valid once tg_assemble or
 * tg_assemble_wait has returned.  out [host]. */
tg_status tg_plan_timing(const tg_load_plan *plan, tg_timing *out);

/* Frees the plan.  If a load begun with it is still in flight (tg_assemble_async /
 * _begin without _wait), the call first waits for the streams and gives the
 * load up as a failed tg_assemble_wait would. */
void tg_plan_free(tg_load_plan *plan);

/*
 * Carry out a plan.  (Section 3.1: load the missing tensors, update the
 * Tensor Mapping, return the GPU address of every tensor; Section 4: tensor
 * transfers are grouped into large copies.)
 *
 * If the plan moves resident tensors, the moves run first on stream_gather,
 * as copy launches whose reads and writes never meet (a stretch that shifts
 * by less than 32 MiB goes through a 128 MiB staging buffer of the library);
 * stream_h2d waits for them.  Then one gather kernel on stream_gather copies
 * every reused tensor into its slot (none in alias mode); at the same time
 * the missing tensors are copied from the model's pinned host buffer with
 * hipMemcpyAsync on stream_h2d (copies that are adjacent on both sides are
 * merged into one).  The call waits for both streams, then commits: evicted
 * rows disappear, moved rows change address, slots become allocated regions,
 * one Tensor Mapping row per new slot is added (aliased rows gain an owner),
 * the model's rows count as in use, the generation advances.
 * out_dev_ptrs [host], if not NULL, receives n_tensors [device] addresses.
 * With TG_ASSEMBLE_VERIFY every slot is fingerprinted on stream_gather before
 * committing -- what the gather wrote right after the gather, the transferred
 * tensors in up to four batches of decreasing size (one per 64 MiB of transfer
 * at most), each as soon as its copies have landed, so that only the last,
 * smallest batch's fingerprint is left when the transfer ends (a transfer
 * below 64 MiB is waited for by the host instead) --
 * and TG_ERR_CORRUPT is returned, without committing, if any differs from its
 * descriptor.  Tensors that the plan moved are fingerprinted at their new
 * addresses too, against their rows of the Tensor Mapping; one that no longer
 * matches (it was damaged before or by the move) also ends the call with
 * TG_ERR_CORRUPT, and its row is removed so that it is never offered for reuse
 * again (unless a running model still uses it).
 * When the call fails after it has started to write (TG_ERR_CORRUPT,
 * TG_ERR_HIP), it first waits for both streams.  A plan without evictions and
 * moves has only written into free regions: the pool is as before and the plan
 * may be assembled again.  Otherwise the plan is given up as by tg_abandon.
 * TG_ERR_STALE if the pool's generation is not the plan's.  A plan can be
 * assembled once.  The two streams may be the same stream.
 */
tg_status tg_assemble(tg_pool *pool, tg_load_plan *plan, uint32_t flags, void *stream_gather,
                      void *stream_h2d, void **out_dev_ptrs);

/*
 * tg_assemble with its arguments in a struct, and one more: a second stream
 * for the host-to-device copies.  With use_second_h2d_stream != 0 the copies
 * are dealt alternately over stream_h2d and stream_h2d_second, so that one
 * starts while the other is still running (a copy costs about 10 us to start
 * on its stream; Section 4 groups small transfers for the same reason).  The
 * second stream obeys the same rules as the first: it waits for the moves, its
 * copies are part of the verification batches, and the call waits for it
 * before it returns.  It is ignored if it equals one of the other two streams
 * or if those two are the same stream.  flags as for tg_assemble.
 */
typedef struct {
    uint32_t flags;
    uint32_t use_second_h2d_stream;
    void    *stream_gather;
    void    *stream_h2d;
    void    *stream_h2d_second;
} tg_assemble_args;
tg_status tg_assemble_ex(tg_pool *pool, tg_load_plan *plan, const tg_assemble_args *args,
                         void **out_dev_ptrs);

/*
 * The same load in steps that do not block.  (Section 3.1 has two sources
 * for what the Tensor Mapping does not hold, a cache in CPU memory and the
 * storage behind it; Section 3.4, Eq. 3: filling the cache and emptying it
 * into the GPU go on at the same time.)
 *
 * tg_assemble_async  enqueues everything tg_assemble_ex does -- moves, the
 *     gather, every host-to-device copy from the plan's host image, the
 *     fingerprints of a verifying load -- and returns without waiting for the
 *     device.  The plan must have a host image if it transfers anything.
 * tg_assemble_begin  enqueues the part that needs no host bytes: moves, the
 *     gather, and their fingerprints.  The missing tensors are then handed
 *     over with tg_assemble_feed, in any order and any number of pieces, from
 *     wherever in pinned memory they happen to be: a Model Cache smaller than
 *     the model is refilled between feeds.  The plan's host image, if it has
 *     one, is not touched.
 * tg_assemble_feed   seg_base [pinned host] .. + seg_bytes holds the bytes of
 *     the n tensors listed in rows [host]: tensor rows[i].tensor (an index
 *     into the model's tensor list; it must be a TG_OP_H2D row of the plan
 *     that has not been fed yet) starts at seg_base + rows[i].seg_off.  Their
 *     copies are enqueued like tg_assemble's (merged where adjacent, dealt
 *     over the two transfer streams, small ones through the gather kernel on
 *     stream_gather, fingerprinted in batches as they land if the load
 *     verifies) and the call returns.  *ticket [host], if not NULL, receives
 *     a number for tg_assemble_feed_wait.  TG_ERR_INVALID for a row that is
 *     out of range, not a transfer, fed twice, or that reaches past seg_bytes;
 *     a feed refused for its rows enqueues nothing and the load goes on.
 * tg_assemble_feed_wait  blocks until the device has read everything the
 *     feed with that ticket reads from its segment, after which the caller
 *     may overwrite the segment (with the next piece of the model).
 * tg_assemble_wait   waits for the streams, checks the fingerprints of a
 *     verifying load, commits and fills out_dev_ptrs exactly as tg_assemble
 *     does, and ends the load.  TG_ERR_INVALID, after waiting, if a missing
 *     tensor was never fed; then, and after any other failure, the load is
 *     given up as described for tg_assemble.
 * One load at a time may be in flight per pool; while it is, the pool accepts
 * tg_plan, tg_reuse_size and the read-outs, and refuses commit, abandon,
 * release and a second begin with TG_ERR_INVALID.  Any of these calls that
 * fails after work was enqueued waits for the streams, gives the load up and
 * ends it; the plan can then only be freed.  Loads on different pools are
 * independent and may run from different threads at the same time.
 */
typedef struct {
    uint32_t tensor;          /* index into the model's tensor list */
    uint32_t reserved;        /* must be 0 */
    uint64_t seg_off;         /* where the tensor's bytes start inside the segment */
} tg_feed_row;
tg_status tg_assemble_async(tg_pool *pool, tg_load_plan *plan, const tg_assemble_args *args);
tg_status tg_assemble_begin(tg_pool *pool, tg_load_plan *plan, const tg_assemble_args *args);
tg_status tg_assemble_feed(tg_pool *pool, tg_load_plan *plan, const void *seg_base, uint64_t seg_bytes,
                           const tg_feed_row *rows, uint32_t n, uint32_t *ticket);
tg_status tg_assemble_feed_wait(tg_pool *pool, tg_load_plan *plan, uint32_t ticket);
tg_status tg_assemble_wait(tg_pool *pool, tg_load_plan *plan, void **out_dev_ptrs);

/*
 * Commit a plan's metadata without enqueuing any copy, for a caller that
 * fills the slots itself (or only wants the bookkeeping).  Same checks and
 * same effect on the Region List and Tensor Mapping as tg_assemble.
 */
tg_status tg_commit(tg_pool *pool, tg_load_plan *plan, void **out_dev_ptrs);

/*
 * Give up a plan after its evictions and moves have happened to the bytes in
 * the pool but its slots could not be filled (what tg_assemble does when it
 * fails half way; for a tg_commit caller that moves the bytes itself).  The
 * evicted rows disappear and the moved rows change address as in a commit
 * (Section 3.2: an evicted tensor's region may have been overwritten, a merged
 * tensor lies at its new address); the slots meant for the model are free
 * regions again; the model gains no rows; the generation advances and the plan
 * is consumed.  TG_ERR_STALE / TG_ERR_INVALID as for tg_commit.
 */
tg_status tg_abandon(tg_pool *pool, tg_load_plan *plan);

/*
 * The model instance ends.  (Section 3.1: tensors of inactive models stay
 * resident and reusable until evicted.)  flags == 0: the model's rows no
 * longer count as in use by it; their bytes stay and keep matching.
 * TG_RELEASE_EVICT: the model also gives up its rows; those that no other
 * model owns are removed and their regions freed and merged with free
 * neighbours.  TG_ERR_NOTFOUND if the pool holds nothing of model_id.
 */
tg_status tg_release(tg_pool *pool, uint64_t model_id, uint32_t flags);

/*
 * Eviction-cost parameters of a model (Eq. 2): miss_prob = p_m, the
 * probability that a tensor of the model is missed once evicted; load_bw =
 * b_m, the bandwidth it would be reloaded at; alpha = alpha_m, the model's
 * latency sensitivity (1 by default, smaller for tolerant models).  May be set
 * before the model is ever loaded; unset models use 1, 1, 1.  How p_m is
 * estimated is the caller's policy (the paper does not fix it).
 * TG_ERR_INVALID unless miss_prob >= 0, load_bw > 0, alpha >= 0.
 */
tg_status tg_set_model_cost(tg_pool *pool, uint64_t model_id, double miss_prob, double load_bw,
                            double alpha);

/*
 * Bytes of `model` that a load would not have to transfer: the sum of nbytes
 * over tensors whose key is resident (S' of the load-time estimate, Eq. 3;
 * the quantity the affinity scheduler of Section 3.4 asks each worker for).
 * est_load_s, if not NULL, receives (S - S') / link_bytes_per_s.
 */
tg_status tg_reuse_size(const tg_pool *pool, const tg_model_desc *model, double link_bytes_per_s,
                        uint64_t *reuse_bytes, double *est_load_s);

/*
 * Page-locked host memory for a Model Cache image (Section 3.1 loads missing
 * tensors from the CPU-side Model Cache; the copy engine needs it pinned).
 * *out [pinned host] receives nbytes of memory that is also mapped into the
 * device's address space.  TG_ERR_NOMEM when the host or the driver's pinned
 * limit is exhausted.  tg_host_free(NULL) is accepted.
 */
tg_status tg_host_alloc(uint64_t nbytes, void **out);
tg_status tg_host_free(void *p);

/* The address under which kernels see a piece of pinned host memory (its
 * device mapping): what to put into a tg_span or tg_pair that should read the
 * Model Cache in place, over the host link.  pinned [pinned host] may point
 * anywhere inside an allocation of tg_host_alloc (or any page-locked, mapped
 * allocation).  TG_ERR_INVALID if the memory is not mapped for the device. */
tg_status tg_host_device_ptr(const void *pinned, void **out_dev);

/* Frees the library's device and pinned scratch.  Safe to call twice. */
void tg_shutdown(void);

/* Static, human-readable name of a status. */
const char *tg_strerror(tg_status s);

#ifdef __cplusplus
}
#endif
#endif /* TANGRAM_H */
