/*
 * rose_delta.h -- C ABI of the MI355X (gfx950) sparse weight-delta library.
 *
 * The library implements the data-parallel part of the cross-cluster weight
 * transfer engine of ROSE (Sec. 4.2): the sender compares the previous and the
 * updated bf16 parameters, keeps only the changed elements in COO form
 * ("Sparsity-aware Weight Transfer"; App. F calls the step D2S), already split
 * by the receiver's tensor-parallel layout ("Shard-aware Weight Transfer":
 * sharded dimension -> per-rank slice ranges), and every receiver applies its
 * own part onto its resident previous weights (App. F: S2D).
 *
 * Conventions
 *   - Every pointer is named host or device below.  The library owns only the
 *     plan handle (and device tables hanging off it); every tensor, bucket,
 *     pointer table and workspace is caller-owned device memory that must stay
 *     valid until the work queued on `stream` has finished.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     encode / apply / dense_copy / bw_probe only queue work and return; they do
 *     not synchronise and do not allocate after the plan's first use on a device
 *     (rose_plan_upload makes that first use explicit).
 *   - A plan is used on ONE device: the first device call on it (or rose_plan_upload)
 *     binds it to the device that is current then; on any other device the calls
 *     return ROSE_ERR_ARG.  Make one plan per device.
 *   - Errors that the host can see are returned before anything is queued.
 *     No exception crosses this boundary.  The library keeps no state outside plan
 *     handles, except the built-in scratch array of rose_delta_encode_static (one
 *     per device, see there).
 *   - Weights are 16-bit patterns (bf16).  "Changed" means the two patterns
 *     differ; an entry carries the new pattern and applying it overwrites.
 *   - Entry coordinates are int32 flat indices local to the destination shard's
 *     copy of one tensor; model-wide positions, offsets and counts are int64.
 */
#ifndef ROSE_DELTA_H
#define ROSE_DELTA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ROSE_MAX_TP 16        /* largest destination tensor-parallel degree */
#define ROSE_MAX_SECTIONS 4   /* largest number of stacked sections of a fused tensor */

typedef enum {
    ROSE_OK = 0,
    ROSE_ERR_ARG = 1,         /* null pointer, index out of range, bad enum value */
    ROSE_ERR_SHAPE = 2,       /* a sharded dimension is not divisible by tp, sections do not add up */
    ROSE_ERR_CAPACITY = 3,    /* a bucket was too small (see rose_bucket_check) */
    ROSE_ERR_ALIGN = 4,       /* a bucket or workspace pointer is not aligned as required */
    ROSE_ERR_HIP = 5,         /* a HIP runtime call failed (no GPU, launch failure), or an encode launch gave up */
    ROSE_ERR_UNSUPPORTED = 6, /* a destination shard's local tensor has 2^31 or more elements, tp > ROSE_MAX_TP */
    ROSE_ERR_SCRATCH = 7      /* rose_delta_encode_static: the plan was not uploaded to this device, or it needs
                                 more scratch than the built-in array holds */
} rose_status;

/* How the receiver's layout cuts a row-major (rows, cols) tensor into tp shards. */
typedef enum {
    ROSE_REPLICATED = 0,  /* every shard holds the whole tensor (norm weights); its entries go
                             to every bucket */
    ROSE_SPLIT_ROWS = 1,  /* dim 0 in tp equal blocks: column-parallel [out,in] matrices, vocabulary */
    ROSE_SPLIT_COLS = 2,  /* dim 1 in tp equal blocks: row-parallel matrices (o_proj, down_proj) */
    ROSE_FUSED_ROWS = 3   /* dim 0 is a stack of sections (Q;K;V or gate;up), each cut in tp equal
                             blocks; shard d holds [sec0_d; sec1_d; ...] */
} rose_rule;

typedef enum {
    ROSE_BF16 = 0,        /* the new weights are bf16 patterns */
    ROSE_FP32_RNE = 1     /* the new weights are fp32 masters, rounded to bf16 (nearest, ties to even,
                             NaN quieted) inside the kernel before they are compared */
} rose_src_dtype;

typedef struct {
    int64_t rows, cols;                            /* full (unsharded) shape; 1-D tensors: rows = 1 */
    int32_t rule;                                  /* rose_rule */
    int32_t n_sections;                            /* ROSE_FUSED_ROWS only: 1..ROSE_MAX_SECTIONS */
    int64_t section_rows[ROSE_MAX_SECTIONS];       /* rows of each section, sum = rows */
    int32_t src_groups;                            /* ROSE_FUSED_ROWS only, sender side: 0 = the sender keeps
                                                      the sections stacked like the destination; G > 0 = it
                                                      keeps them interleaved by G head groups (for each group
                                                      its rows of section 0, then of section 1, ...: the usual
                                                      training-side layout of a fused QKV matrix) and senders
                                                      split that layout in tp_src equal row blocks (whole
                                                      groups).  Every section and tp_src must divide by G
                                                      resp. into it. */
    int32_t layer;                                 /* pipeline plans (rose_shard_plan_create_pp) only: decoder layer
                                                      0 .. n_layers-1 the tensor belongs to, ROSE_LAYER_FIRST for
                                                      tensors in front of the layers (embedding), ROSE_LAYER_LAST
                                                      for those behind them (final norm, head); ignored otherwise */
} rose_tensor_desc;
#define ROSE_LAYER_FIRST (-1)
#define ROSE_LAYER_LAST (-2)

typedef struct rose_plan rose_plan;

/*
 * One destination shard's COO data (Sec. 4.2, sparsity-aware transfer: the COO data is split by the
 * receiver's parallel layout).  The struct lives in host memory; all four arrays are device memory.
 *   idx      [capacity] int32 local indices, 16-byte aligned
 *   val      [capacity] new 16-bit patterns, 16-byte aligned
 *   seg_off  [n_tensors + 1] int64, 8-byte aligned: after encode, the entries of tensor t are
 *            idx/val[seg_off[t] .. seg_off[t+1]), in ascending local index; seg_off[n_tensors]
 *            is the exact number of entries the shard needs, also when it exceeds capacity
 *            (then entries at positions >= capacity were dropped, nothing was written out of
 *            bounds, and the bucket must not be applied).
 */
typedef struct {
    int32_t *idx;
    uint16_t *val;
    int64_t capacity;
    int64_t *seg_off;
} rose_bucket;

/*
 * shard_plan (Sec. 4.2 "Shard-aware Weight Transfer"): per tensor, the rule and the per-rank
 * slice ranges, turned into the tables the kernels walk.  Pure host work, no GPU needed.
 * `tensors` (host, copied) lists the model's tensors in bucket order.  Errors: ROSE_ERR_ARG,
 * ROSE_ERR_SHAPE, ROSE_ERR_UNSUPPORTED.  On success *out is a handle to free with
 * rose_shard_plan_destroy; it is immutable and may be used from several threads.
 */
rose_status rose_shard_plan_create(const rose_tensor_desc *tensors, int32_t n_tensors, int32_t tp,
                                   rose_plan **out);
/*
 * The same for a sender that holds only its own slice of every tensor (Sec. 4.2: per-rank slice
 * ranges on both sides; training and serving may use different degrees): the sender is rank
 * src_rank of tp_src under the SAME rule per tensor, and old / new pointers given to
 * rose_delta_encode point at its slices (rose_plan_src_numel elements each, laid out like a
 * destination shard of degree tp_src).  Each element goes to the destination shard that holds it,
 * at that shard's local index; a destination is only reached where the two slice ranges overlap.
 * A replicated tensor is held by every sender and sent by exactly one: sender (ordinal mod
 * tp_src); the others' pointers for it are not read by rose_delta_encode (with ROSE_ENCODE_REFRESH
 * they are: every sender refreshes its own copy; rose_plan_tensor_is_read tells).  The tp_src senders' buckets for one
 * destination are disjoint and may be applied in any order.  tp_src = 1, src_rank = 0 is
 * rose_shard_plan_create.  rose_dense_copy with such a plan copies the part of the destination
 * shard that the sender holds.  Errors as above; both degrees must divide the split dimensions.
 */
rose_status rose_shard_plan_create_src(const rose_tensor_desc *tensors, int32_t n_tensors, int32_t tp,
                                       int32_t tp_src, int32_t src_rank, rose_plan **out);
/*
 * The same with pipeline stages on both sides (Sec. 4.2 "Shard-aware Weight Transfer": TP and PP on the
 * training and on the serving side, e.g. TP 8 x PP 2 feeding TP 4).  `tensors` lists the WHOLE model in
 * one order that every sender and receiver shares, each tensor naming its layer; a side with pp stages
 * deals the n_layers layers to them in equal consecutive groups (pp must divide n_layers), ROSE_LAYER_FIRST
 * tensors go with stage 0, ROSE_LAYER_LAST tensors with the last stage.
 *   sender    rank src_rank of tp_src in stage stage_src of pp_src: it holds (and encode reads) only the
 *             tensors of its stage; the pointer-table entries of all other tensors are never read.
 *   receiver  pp_dst stages of tp shards each.  There are tp * pp_dst buckets (at most ROSE_MAX_TP):
 *             bucket b = stage * tp + shard receives the tensors of that stage.  Wherever this header says
 *             "shard d" of a plan (rose_delta_encode's bucket array, rose_delta_apply, rose_dense_copy,
 *             rose_bucket_pack, an object's shard word, the queries), a pipeline plan takes the bucket number.
 * Tensor numbers stay model-wide everywhere: seg_off has n_tensors + 1 entries in every bucket (segments
 * of tensors that the bucket's stage does not hold are empty), a receiver's dst_ptrs table has
 * n_tensors entries of which only its own stage's are read, and a transport object carries the
 * model-wide segment table, so a receiver whose stage split differs from the sender's places every
 * entry by (tensor number, local index) alone.  rose_plan_local_numel is 0 for a tensor the bucket's
 * stage does not hold, rose_plan_src_numel is 0 for one the sender does not hold.
 * pp_src = pp_dst = 1 is rose_shard_plan_create_src.  Errors as above; ROSE_ERR_SHAPE if a pp does not
 * divide n_layers, ROSE_ERR_ARG for a layer outside 0 .. n_layers-1, ROSE_ERR_UNSUPPORTED if tp * pp_dst
 * exceeds ROSE_MAX_TP.
 */
rose_status rose_shard_plan_create_pp(const rose_tensor_desc *tensors, int32_t n_tensors, int32_t tp,
                                      int32_t tp_src, int32_t src_rank, int32_t n_layers, int32_t pp_src,
                                      int32_t stage_src, int32_t pp_dst, rose_plan **out);
void rose_shard_plan_destroy(rose_plan *plan);
/*
 * Makes the plan resident on the current device (HOST call; allocates and copies the plan's tables,
 * asks the runtime how many workgroups of each kernel fit, looks up the built-in scratch array) and
 * binds the plan to that device.  The other device calls do this by themselves on first use; call it
 * ahead of time where a later call must not allocate (graph capture, rose_delta_encode_static).
 * Idempotent.  ROSE_ERR_HIP if the runtime fails, ROSE_ERR_ARG if the plan is bound to another device.
 */
rose_status rose_plan_upload(const rose_plan *plan);
/*
 * Caps the number of workgroups of later encode launches with this plan that walk tiles, e.g. to
 * leave compute units to other kernels (0 = no cap, the default; values of 64 or less, or above what
 * the device holds, are ignored).  May be called at any time from any thread; a launch uses the value
 * it finds.
 */
rose_status rose_plan_set_worker_cap(rose_plan *plan, int32_t workers);
/*
 * The order in which the encode kernel's workgroups take tiles (it changes speed only: the buckets
 * are the same bytes either way).  ROSE_TILE_ORDER_SPREAD: a workgroup takes tiles that lie 64 tiles
 * apart, so that the prefix sums across workgroups are ready soonest; best above about 7.5 % of changed
 * elements.  ROSE_TILE_ORDER_NEIGHBOURS: it takes three neighbouring tiles and writes their entries
 * as one run, which shares fewer 64-byte lines of the bucket with other workgroups; best between
 * about 4 and 7.5 %.  ROSE_TILE_ORDER_TIMED: four neighbouring tiles, and the entries are held in the
 * workgroup until a window of time that all workgroups share (they read one clock), so that the
 * memory sees the bucket writes in bursts instead of a steady trickle among the reads; best below
 * about 4 %.  ROSE_TILE_ORDER_AUTO_PICK (the default): the library picks, from the density of the
 * plan's previous launch as far as rose_bucket_check has read it back (until then from the share of
 * the shards that the buckets passed in could hold at most).
 * May be called at any time from any thread; a launch uses the value it finds.
 */
#define ROSE_TILE_ORDER_AUTO_PICK 0
#define ROSE_TILE_ORDER_SPREAD 1
#define ROSE_TILE_ORDER_NEIGHBOURS 2
#define ROSE_TILE_ORDER_TIMED 3
rose_status rose_plan_set_tile_order(rose_plan *plan, int32_t order);
/*
 * The order an encode launch into `buckets` (HOST array of rose_plan_n_buckets structs; only the
 * capacities are read) would use at this moment: the order set, or the library's pick.  Host only.
 * ROSE_ERR_ARG for null pointers.
 */
rose_status rose_plan_pick_tile_order(const rose_plan *plan, const rose_bucket *buckets, int32_t *order);

/* Host queries on a plan (no GPU needed). */
int32_t rose_plan_n_tensors(const rose_plan *plan);
int32_t rose_plan_tp(const rose_plan *plan);
/* number of buckets: tp, or tp * pp_dst for a pipeline plan */
int32_t rose_plan_n_buckets(const rose_plan *plan);
/* stage that holds tensor t on the sending and on the receiving side (each may be NULL) */
rose_status rose_plan_stage_of(const rose_plan *plan, int32_t t, int32_t *stage_src, int32_t *stage_dst);
/* *is_read = 1 if an encode launch with these flags (ROSE_ENCODE_*) dereferences entry t of old_ptrs and
 * new_ptrs: the sender holds the tensor, it is not empty, and the sender sends it or (ROSE_ENCODE_REFRESH)
 * refreshes it.  Entries with 0 may hold anything. */
rose_status rose_plan_tensor_is_read(const rose_plan *plan, int32_t t, uint32_t flags, int32_t *is_read);
/* elements of the model before tensor t (int64 model-wide position of its element 0) */
rose_status rose_plan_tensor_base(const rose_plan *plan, int32_t t, int64_t *global_base);
/* elements of shard d's local copy of tensor t */
rose_status rose_plan_local_numel(const rose_plan *plan, int32_t t, int32_t d, int64_t *numel);
/* elements of the sender's slice of tensor t (the full tensor unless the plan has tp_src > 1) */
rose_status rose_plan_src_numel(const rose_plan *plan, int32_t t, int64_t *numel);
/* flat element g of the sender's slice of tensor t goes to shards d_first .. d_first + n_dest - 1 at
 * local index *local (n_dest = 0: a replicated tensor that another sender sends) */
rose_status rose_plan_map_index(const rose_plan *plan, int32_t t, int64_t g, int32_t *d_first,
                                int32_t *n_dest, int32_t *local);
/* worst-case number of entries this sender produces for bucket d (every element changed) */
rose_status rose_plan_bucket_capacity(const rose_plan *plan, int32_t d, int64_t *max_entries);
/* bytes of device scratch that rose_delta_encode needs (256-byte aligned buffer) */
rose_status rose_plan_workspace_bytes(const rose_plan *plan, size_t *bytes);
/* number of tiles the encode kernel walks (for reporting) */
rose_status rose_plan_n_tiles(const rose_plan *plan, int64_t *n_tiles);

/*
 * delta_encode (Sec. 4.2 "Sparsity-aware Weight Transfer", App. F D2S): one pass over the
 * previous and the new weights that writes all tp buckets.
 *   old_ptrs, new_ptrs  DEVICE arrays of n_tensors device pointers to the full tensors
 *                       (row-major; bf16, or fp32 for new when new_dtype = ROSE_FP32_RNE).
 *                       Tensors aligned to 16 bytes take the 128-bit load path; others still
 *                       work, more slowly.  Both are only read.
 *   buckets             HOST array of rose_plan_n_buckets bucket structs (tp of them; tp * pp_dst for a
 *                       pipeline plan); their device arrays are written.
 *   workspace           DEVICE scratch of at least rose_plan_workspace_bytes, 256-byte aligned;
 *                       contents before the call do not matter; calls that share a workspace
 *                       must be ordered on one stream.
 * Returns ROSE_ERR_ARG / ROSE_ERR_ALIGN / ROSE_ERR_HIP without queuing anything.  A bucket
 * that is too small is not an error of this call: see rose_bucket_check.
 *
 * The kernel's workgroups wait on each other's tile counts.  The wait is bounded: if a count does
 * not arrive within a few seconds the launch is marked as failed, every workgroup still exits,
 * seg_off[n_tensors] of every bucket is set to -1, rose_bucket_check returns ROSE_ERR_HIP and
 * rose_delta_apply of such a bucket does nothing.
 *
 * The grid is sized so that all of its workgroups fit on the device at once, and progress is
 * argued for that case.  Kernels of other streams that hold compute units while the launch runs
 * only delay it as long as they end; two encode launches running at the same time on one device
 * (different streams, different workspaces) can starve each other until the bounded wait gives up:
 * order encode launches of one device on one stream.
 *
 * rose_plan_set_worker_cap limits the workgroups that walk tiles.  After a launch the 32-bit words 2
 * and 3 of the workspace hold diagnostic counts (how often a workgroup received two tickets of one group of blocks in a row;
 * how often it counted a ticket's remaining tiles ahead of a wait, which happens where more than
 * about a third of the elements change).
 */
rose_status rose_delta_encode(const rose_plan *plan, const void *const *old_ptrs,
                              const void *const *new_ptrs, int32_t new_dtype,
                              const rose_bucket *buckets, void *workspace, size_t workspace_bytes,
                              void *stream);

/*
 * delta_encode with sender refresh (Sec. 4.2: the sender keeps W_{t-1} resident and makes it
 * current for the next step): the same buckets as rose_delta_encode, and afterwards every old
 * tensor the sender holds equals the new one as bf16 (for fp32 input: its round-to-nearest-even
 * cast), so that the same old tensors serve the next step while the new ones may be overwritten by
 * the trainer.  Only the 16-byte vectors that contain a change are written (whole replicated
 * tensors, which are small, are copied by a second kernel once every destination has read them;
 * that includes the replicated tensors a sender holds without sending them, so their old and new
 * pointers must be valid here although rose_delta_encode never reads them).
 * old_ptrs' tensors are WRITTEN; everything else as rose_delta_encode.  If the launch gives up
 * (see above) or a bucket overflows, old is already partly refreshed and the dropped entries
 * cannot be produced again from it: size buckets for the worst case when using this call, or
 * keep the new weights until rose_bucket_check has passed.
 */
rose_status rose_delta_encode_refresh(const rose_plan *plan, void *const *old_ptrs,
                                      const void *const *new_ptrs, int32_t new_dtype,
                                      const rose_bucket *buckets, void *workspace, size_t workspace_bytes,
                                      void *stream);

/*
 * Arithmetic payload (Sec. 4.2 states the update as W_t = W_{t-1} + dW_t; a variant that takes this
 * literally.  The paper fixes no element format: the rule below is this library's).
 * An entry of a bucket written with ROSE_ENCODE_ARITH carries val = bf16(new - old), rounded to
 * nearest even, if that difference is a number and bf16(old + val) is exactly the new pattern; the
 * receiver then ADDS val to its resident value (same rounding).  Where that does not hold (large
 * jumps, a change of a zero's sign, infinities and NaNs) the entry carries the new pattern instead
 * and bit 31 of its index is set (the index is negative); the receiver overwrites.  Index order,
 * counts and seg_off are the same as for the default payload, so buckets have the same size.
 * With the escape the variant is lossless for all patterns, PROVIDED the receiver's copy holds
 * exactly the sender's old weights: unlike the default payload, applying a bucket twice, or onto
 * another state, gives wrong weights.  Subnormal values are kept, not flushed.
 *
 * rose_delta_encode_ex   rose_delta_encode with flags: ROSE_ENCODE_REFRESH as
 *                        rose_delta_encode_refresh (old tensors are written), ROSE_ENCODE_ARITH
 *                        arithmetic payloads; flags = 0 is rose_delta_encode.  Unknown bits:
 *                        ROSE_ERR_ARG.
 * rose_delta_apply_ex    rose_delta_apply for a bucket of the given payload kind.
 * rose_bucket_pack_ex    rose_bucket_pack that records the payload kind in the object's header
 *                        (u32 at byte 32); rose_object_apply reads it there.
 */
#define ROSE_ENCODE_REFRESH 1u
#define ROSE_ENCODE_ARITH 2u
#define ROSE_PAYLOAD_NEW 0
#define ROSE_PAYLOAD_ARITH 1
rose_status rose_delta_encode_ex(const rose_plan *plan, void *const *old_ptrs, const void *const *new_ptrs,
                                 int32_t new_dtype, uint32_t flags, const rose_bucket *buckets,
                                 void *workspace, size_t workspace_bytes, void *stream);
rose_status rose_delta_apply_ex(const rose_plan *plan, int32_t d, const rose_bucket *bucket, int32_t payload,
                                void *const *dst_ptrs, void *stream);

/*
 * rose_delta_encode_ex for callers that cannot allocate or bring a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  The scratch that the kernels need
 * (tile and block descriptors, ticket counter, abort flag) lives in an array built into the library,
 * ROSE_STATIC_SCRATCH_BYTES per device, held from the library's load to the end of the process.
 * The call allocates nothing and frees nothing; it queues the same kernels as rose_delta_encode_ex and
 * the buckets come out identical.
 *   - the plan must be resident on the current device already (rose_plan_upload, or any earlier
 *     device call on it): otherwise ROSE_ERR_SCRATCH, nothing queued;
 *   - rose_plan_workspace_bytes(plan) must not exceed ROSE_STATIC_SCRATCH_BYTES (about 6 million
 *     tiles, i.e. 50 G elements): otherwise ROSE_ERR_SCRATCH, nothing queued;
 *   - every call on a device shares that device's array, which keeps the previous call's contents
 *     (the launch clears what it uses first): calls that overlap in time on one device race, whatever
 *     their streams or plans.  Order them on one stream.
 */
#define ROSE_STATIC_SCRATCH_BYTES (48u << 20)
rose_status rose_delta_encode_static(const rose_plan *plan, void *const *old_ptrs, const void *const *new_ptrs,
                                     int32_t new_dtype, uint32_t flags, const rose_bucket *buckets, void *stream);

/*
 * delta_apply (Sec. 4.2, sparsity-aware transfer: a receiver applies its own shard only; App. F S2D): writes every
 * entry's value at its local index of shard d's resident copies.
 *   bucket    HOST struct, device arrays as written by rose_delta_encode for shard d
 *   dst_ptrs  DEVICE array of n_tensors device pointers to shard d's local tensors
 *             (rose_plan_local_numel elements each, 2-byte aligned at least)
 * Entries at positions >= capacity (an overflowed bucket) are not applied, nor are entries whose
 * index lies outside their tensor.
 * The kernel reads and rewrites whole 64-byte pieces of a destination tensor around the entries
 * it applies (never a byte outside the tensor): nothing else may write the destination tensors
 * while the call runs.  The first device call on a plan (encode, apply or dense copy) uploads the
 * plan's tables with hipMalloc / hipMemcpy; later calls allocate nothing.
 */
rose_status rose_delta_apply(const rose_plan *plan, int32_t d, const rose_bucket *bucket,
                             void *const *dst_ptrs, void *stream);

/*
 * Dense path (Sec. 4.2 "Shard-aware Weight Transfer" without sparsity; the comparison the
 * Sec. 6.3 crossover is measured against): dst = shard d's slice of the new weights.
 * Pointer tables as above.
 */
rose_status rose_dense_copy(const rose_plan *plan, int32_t d, const void *const *new_ptrs,
                            int32_t new_dtype, void *const *dst_ptrs, void *stream);

/*
 * Synchronises `stream`, reads seg_off[n_tensors] of the bucket back and returns
 * ROSE_ERR_CAPACITY if it exceeds capacity.  *required (host, may be NULL) gets the count.
 * The plan remembers the density that the count implies (see rose_plan_set_tile_order).
 */
rose_status rose_bucket_check(const rose_plan *plan, const rose_bucket *bucket, void *stream,
                              int64_t *required);

/*
 * Transport objects (Sec. 4.2 "Asynchronous Weight Transfer": senders push fixed-size buckets to
 * a relay, receivers pull the ones their metadata names).  A destination's entry stream is cut
 * into objects that describe themselves, so that each can be applied alone, in any order.
 * Layout of an object holding n entries of a plan with T tensors (little endian, this library's
 * own format; all of it device memory, 16-byte aligned):
 *     0  u32 magic ROSE_OBJECT_MAGIC, u32 version 1, i32 shard, i32 T
 *    16  i64 first_entry (position of the object's first entry in the shard's stream), i64 n
 *    32  u32 payload kind (0 new patterns, 1 arithmetic payloads), then zero up to 64
 *    64  i64 seg_off[T + 1]: the entries of tensor t are [seg_off[t], seg_off[t+1]) of THIS object
 *     A  i32 idx[n], A = 64 + 8 (T + 1) rounded up to 16
 *     B  u16 val[n], B = A + 4 n rounded up to 16; size = B + 2 n rounded up to 16 (slack is zero)
 *
 * rose_object_bytes   size of an object with n_entries.
 * rose_bucket_pack    writes entries [first_entry, first_entry + n_entries) of bucket d (as left by
 *                     rose_delta_encode) into `object`.  The host checks sizes (ROSE_ERR_CAPACITY if
 *                     object_bytes is too small); the range is checked against the bucket's true
 *                     total on the device: a range beyond it yields an object with a zero magic,
 *                     which nobody applies.
 * rose_object_apply   checks the object on the device and applies the entries to the shard's
 *                     tensors; an object that fails the check changes nothing.  Checked: the header
 *                     (magic, version, shard, T, sizes against object_bytes), the segment table (starts
 *                     at 0, never decreases, ends at n) and, in a pass over all indices, that they
 *                     ascend strictly inside every segment (the apply kernel's ownership of 64-byte
 *                     pieces relies on that order; an index outside its tensor is dropped as in
 *                     rose_delta_apply).  The verdict travels through one of 4096 words of the plan's
 *                     device memory, taken in turn: more than 4096 object applies of one plan in
 *                     flight at once may take each other's verdicts.  Same rule as rose_delta_apply
 *                     about concurrent writers of the destination.
 * rose_object_check   synchronises `stream`, reads the header back and returns ROSE_ERR_ARG for a
 *                     malformed object; shard / first_entry / n_entries / payload kind (host, each
 *                     may be NULL).
 */
#define ROSE_OBJECT_MAGIC 0x45534F52u
rose_status rose_object_bytes(const rose_plan *plan, int64_t n_entries, size_t *bytes);
rose_status rose_bucket_pack(const rose_plan *plan, int32_t d, const rose_bucket *bucket, int64_t first_entry,
                             int64_t n_entries, void *object, size_t object_bytes, void *stream);
rose_status rose_bucket_pack_ex(const rose_plan *plan, int32_t d, const rose_bucket *bucket, int32_t payload,
                                int64_t first_entry, int64_t n_entries, void *object, size_t object_bytes,
                                void *stream);
rose_status rose_object_apply(const rose_plan *plan, const void *object, size_t object_bytes,
                              void *const *dst_ptrs, void *stream);
rose_status rose_object_check(const rose_plan *plan, const void *object, size_t object_bytes, void *stream,
                              int32_t *shard, int64_t *first_entry, int64_t *n_entries, int32_t *payload);

/*
 * Bandwidth probe, for measuring what HBM delivers beside the kernels above: copies `bytes`
 * (a multiple of 16) from src to dst (device, 16-byte aligned); with dst = NULL it only reads
 * src; *sink (device, 8 bytes, required in that mode) exists so that the reads cannot be dropped
 * and is incremented for the rare lane whose checksum hits a fixed constant.
 */
rose_status rose_bw_probe(const void *src, void *dst, size_t bytes, uint64_t *sink, void *stream);

/*
 * Mixed probe: the memory traffic of a delta_encode launch without its work, to measure what HBM
 * delivers for that mix of reads and writes.  Reads read_bytes (a multiple of ROSE_PROBE_CHUNK)
 * from each of src_a and src_b in chunks of ROSE_PROBE_CHUNK bytes and writes
 * write_bytes_per_chunk (a multiple of 16, at most ROSE_PROBE_CHUNK) per chunk to dst, contiguous
 * across chunks: dst needs (read_bytes / ROSE_PROBE_CHUNK) * write_bytes_per_chunk bytes.  All
 * device memory, 16-byte aligned; sink as in rose_bw_probe.
 */
#define ROSE_PROBE_CHUNK 16384
rose_status rose_bw_probe_mixed(const void *src_a, const void *src_b, void *dst, size_t read_bytes,
                                size_t write_bytes_per_chunk, uint64_t *sink, void *stream);
/*
 * The same traffic with the writes bunched in time: a workgroup writes the output of the chunks it
 * has read only in the windows of time that ROSE_TILE_ORDER_TIMED uses (or when 64 chunks are due),
 * to measure what the memory gains from taking the writes in bursts.  Same arguments and errors.
 */
rose_status rose_bw_probe_mixed_timed(const void *src_a, const void *src_b, void *dst, size_t read_bytes,
                                      size_t write_bytes_per_chunk, uint64_t *sink, void *stream);

/*
 * Line probe: what HBM delivers for delta_apply's access pattern without any of its work.  Reads,
 * changes and writes back a pseudo-random subset of the 64-byte lines of dst (device, 64-byte aligned,
 * `bytes` a multiple of 64): line i is touched if a fixed hash of i is below touched_per_2_32, i.e.
 * about that fraction / 2^32 of the lines, independently.  Every 32-bit word at the start of a
 * 16-byte part of a touched line is incremented; nothing else changes.
 */
rose_status rose_bw_probe_lines(void *dst, size_t bytes, uint32_t touched_per_2_32, void *stream);

const char *rose_status_str(rose_status s);

#ifdef __cplusplus
}
#endif
#endif /* ROSE_DELTA_H */
