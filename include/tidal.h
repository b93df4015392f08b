/*
 * tidal.h -- C ABI of libtidal: GPU-side materialisation of an LLM function's state
 * onto a resident template, and per-invocation LoRA attach / swap, for AMD MI355X
 * (gfx950).
 *
 * Framing (arXiv 2503.06421).  A *template* is pre-initialised function state kept in
 * GPU memory from which invocations start (Sec. 1; Sec. 2.3 "template-start").  Its
 * weights are laid out in the traced access order (Sec. 4.2), streamed host->GPU
 * asynchronously in that order from a pinned host pool (Sec. 5.2 "Efficient overlapping
 * with correctness ensuring"), with many small tensors merged into fewer copies (Sec. 6
 * "Tailored memory pool in template server").  Request-specific state -- a LoRA
 * adapter -- is initialised per invocation on top of the reused static state (Sec. 5.2
 * "Adaptive template state reusing"), and while a function is kept alive only that
 * dynamic part is redone (Sec. 5.2 "Keep-alive of dynamic function").
 *
 * Conventions.
 *   - Every pointer is tagged [host] or [device].  No C++ or framework types cross
 *     the boundary; streams are hipStream_t passed as void* (NULL = the null stream).
 *   - The caller owns the device arena, the device memory of resident adapters and the
 *     streams.  The library owns the handle, its pinned bounce buffers and its events.
 *   - Host source / adapter pointers are borrowed until the stream work of the call
 *     has completed (tidal_template_sync, or a sync of the streams given).
 *   - Calls are asynchronous with respect to the host and ordered on the given
 *     streams; in addition every LoRA / fork call waits (on the GPU) for the template's
 *     last materialisation and every materialisation for its last LoRA call, whatever
 *     streams those used.  LoRA calls among themselves are ordered only by their streams:
 *     issue them on one stream or order them yourself.  One thread at a time per template;
 *     different templates may be driven from different threads at the same time.
 *   - Adapters and forks refer to their template: destroy them before it.
 *   - Every int-returning call returns TIDAL_OK (0) or a negative tidal_status;
 *     tidal_last_error() then holds a message (thread-local).  Arguments are validated
 *     before any work is enqueued: a failed call leaves every slot untouched.  Nothing
 *     throws or aborts across the boundary.
 *   - There is no CPU fallback: calls that need the GPU return TIDAL_E_HIP without one.
 *
 * Template slots hold bf16, row-major, rows = output features, cols = input features.
 */
#ifndef TIDAL_H_
#define TIDAL_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tidal_template tidal_template;   /* opaque, freed by tidal_template_destroy */
typedef struct tidal_adapter tidal_adapter;     /* opaque, freed by tidal_adapter_destroy  */
typedef struct tidal_fork tidal_fork;           /* opaque, freed by tidal_fork_destroy     */

/* Element types of host sources and LoRA factors.  Structs and calls carry the value in an int32_t
 * field or argument: the width of a C enum is the compiler's choice, that of int32_t is not, and the
 * records are filled in from other languages through this ABI. */
typedef enum { TIDAL_F32 = 0, TIDAL_F16 = 1, TIDAL_BF16 = 2 } tidal_dtype;

typedef enum {
    TIDAL_OK = 0,
    TIDAL_E_INVAL = -1,   /* null / negative / out-of-range argument, unknown dtype, shape mismatch   */
    TIDAL_E_NOMEM = -2,   /* arena, adapter region or caller buffer too small; host allocation failed */
    TIDAL_E_STATE = -3,   /* attach while attached, swap/detach with nothing attached, LoRA on a slot
                             that was never materialised, partial re-materialisation under an adapter */
    TIDAL_E_HIP = -4      /* a HIP runtime call failed (message in tidal_last_error)                  */
} tidal_status;

/* One template slot: a rows x cols bf16 matrix (1-D tensors: rows = 1). */
typedef struct { int64_t rows, cols; } tidal_slot_desc;

/* One tensor to materialise: rows*cols elements of `dtype` at `host`, row-major, dense. */
typedef struct { int32_t slot; int32_t dtype /* a tidal_dtype value */; const void* host; /* [host] borrowed */ } tidal_src;

/* One LoRA target: slot W (out x in) gets W + (alpha/r) * B * A with A (r x in) and
 * B (out x r), row-major, dense, both of `dtype`.  r == 0 or alpha == 0 is valid and
 * leaves W untouched (A and B may then be NULL).  A factor is staged whole, so each of A and
 * B must fit in chunk_bytes (TIDAL_E_INVAL otherwise; with the default 128 MiB that is a rank-64
 * factor of a million columns). */
typedef struct {
    int32_t slot;
    int32_t r;
    float alpha;
    int32_t dtype;        /* a tidal_dtype value */
    const void* A;        /* [host] borrowed */
    const void* B;        /* [host] borrowed */
} tidal_lora_target;

enum {
    /* LoRA kernels accumulate sum_k B[i][k]*A[k][j] as one fp32 fused-multiply-add chain in
     * ascending k on the vector ALUs (bit-reproducible against a sequential definition)
     * instead of the default matrix-core tiles (fp32 accumulation, unspecified order).      */
    TIDAL_FLAG_ORDERED_ACCUM = 1,
    /* tidal_lora_swap runs as two passes over W (unmerge, then merge) instead of one fused
     * pass.  Results are bit-identical; this exists to demonstrate exactly that.              */
    TIDAL_FLAG_TWO_PASS_SWAP = 2,
    /* tidal_materialize records a completion event per slot, for tidal_template_slot_wait.    */
    TIDAL_FLAG_SLOT_EVENTS = 4,
    /* Bracket every convert and LoRA kernel launch with timing events on its stream and add
     * the elapsed times to tidal_stats (tidal_get_stats then waits for those kernels).          */
    TIDAL_FLAG_KERNEL_TIMING = 8,
    /* tidal_materialize enqueues every chunk without waiting, however many there are (by default
     * only a load of up to tidal_config.chunks_ahead chunks is enqueued that way).             */
    TIDAL_FLAG_ASYNC_ENQUEUE = 16,
    /* Issue one hipMemcpyAsync per planned piece: neighbouring pieces are not merged into one
     * copy and tiny tensors are not gathered by the CPU.  For measuring what tensor merging
     * (Sec. 6) buys; results are identical.                                                    */
    TIDAL_FLAG_NO_COPY_MERGE = 32,
    /* tidal_lora_attach / _swap upload and merge an adapter in groups of targets: the factors of
     * all groups cross the link back to back on a stream of the library's own, and the caller's
     * stream packs and merges each group as soon as it has arrived, so that most of the upload
     * hides under the merges (or the other way round).  This needs factors in pinned host memory
     * (pageable ones always take the single pass).  By default the library does it for adapters of
     * 4 MiB or more where its estimate says it pays, with groups sized from link and pass rates it
     * measures with its own events; results are identical to a single pass either way.
     * PIPELINED_UPLOAD: always (two groups or more, whatever the size); SERIAL_UPLOAD: never --
     * everything on the caller's stream, upload first, then one launch per group of equal shapes. */
    TIDAL_FLAG_PIPELINED_UPLOAD = 64,
    TIDAL_FLAG_SERIAL_UPLOAD = 128
};

typedef struct {
    size_t chunk_bytes;        /* source bytes per staged copy unit; 0 = 128 MiB; rounded to 4 KiB;
                                  must be at least 64 KiB                                        */
    int32_t max_rank;          /* largest r accepted; 0 = 64; at most 64                         */
    size_t max_adapter_bytes;  /* size of each of the two in-arena regions that hold the packed
                                  device copy of adapters given by host pointers; 0 = none (then
                                  only resident adapters can be attached)                        */
    int32_t flags;             /* TIDAL_FLAG_*                                                   */
    size_t coalesce_bytes;     /* host tensors smaller than this are gathered by the CPU into a
                                  pinned buffer and shipped as one copy; 0 = 64 KiB              */
    int32_t gather_threads;    /* host threads that copy pageable sources into the pinned buffer
                                  (pieces of 8 MiB or more are split among them); 0 = 4, at most
                                  16.  One thread moves about half of what the link carries.     */
    int32_t chunks_ahead;      /* tidal_materialize enqueues a load of up to this many staged chunks
                                  in one burst and returns (chunks of earlier loads that are still
                                  in flight count against it); in a longer load the calling thread
                                  stays two chunks ahead of the GPU until only this many remain
                                  (a few hundred queued cross-stream waits slow every copy
                                  down, small chunks sooner than large ones).  0 = chunk_bytes /
                                  800 KiB, within 16..160 (160 for 128 MiB chunks); at most 4096. */
} tidal_config;

/* One planned host->device copy unit, as tidal_materialize would issue it (introspection). */
typedef struct {
    int32_t chunk;             /* index of the staged chunk this piece belongs to               */
    int32_t slot;
    int64_t elem_offset;       /* first element of the slot covered by this piece               */
    int64_t elems;
    int64_t src_bytes;         /* bytes read from the host tensor                                */
    int64_t staging_offset;    /* byte offset inside the staging buffer; -1 = copied straight
                                  into the slot (bf16 sources need no conversion)                */
    int32_t gathered;          /* 1 = goes through the CPU-gathered pinned buffer                */
    int32_t reserved;
} tidal_copy_piece;

typedef struct {
    uint64_t h2d_bytes;          /* source bytes sent host->device (tensors and adapters)        */
    uint64_t h2d_copies;         /* hipMemcpyAsync calls issued                                  */
    uint64_t chunks;             /* staged chunks processed                                      */
    uint64_t converted_elems;    /* elements narrowed to bf16 by the convert kernel              */
    uint64_t gathered_bytes;     /* bytes that went through the CPU-gathered pinned buffer       */
    uint64_t rmw_elems;          /* W elements read-modified-written by LoRA kernels             */
    uint64_t lora_launches;      /* LoRA kernel launches                                         */
    double lora_kernel_ms;       /* sum of LoRA kernel durations (TIDAL_FLAG_KERNEL_TIMING)      */
    double convert_kernel_ms;    /* sum of convert kernel durations (TIDAL_FLAG_KERNEL_TIMING)   */
} tidal_stats;

/* Fill *cfg with the defaults named above.  Never fails for non-NULL cfg. */
int tidal_config_default(tidal_config* cfg /* [host] out */);

/* Bytes of device arena tidal_template_create needs: slot area (each slot 256-byte aligned,
 * in the given order -- the access order of Sec. 4.2) + two staging buffers of chunk_bytes
 * + two adapter regions of max_adapter_bytes.  Returns 0 on
 * invalid arguments. */
size_t tidal_template_required_bytes(const tidal_slot_desc* slots /* [host] */, int32_t n,
                                     const tidal_config* cfg /* [host] NULL = defaults */);

/* Create a template over a caller-owned device arena (Sec. 1: the template is function
 * state cached in GPU memory).  Host-only: touches no device memory and makes no HIP call;
 * device resources are created on first use.  dev_arena must be 256-byte aligned and at
 * least tidal_template_required_bytes() long, else TIDAL_E_INVAL / TIDAL_E_NOMEM. */
int tidal_template_create(const tidal_slot_desc* slots /* [host] copied */, int32_t n,
                          void* dev_arena /* [device] borrowed for the template's life */,
                          size_t arena_bytes, const tidal_config* cfg /* [host] NULL = defaults */,
                          tidal_template** out /* [host] out */);

/* Stream the given host tensors into their slots, in the order given (the load order of
 * Sec. 5.2), in chunks of chunk_bytes: pinned (or CPU-gathered) host memory ->
 * hipMemcpyAsync on copy_stream into one of two device staging buffers -> conversion to
 * bf16 (round to nearest even, subnormals kept, NaN quieted) into the slot on
 * compute_stream; bf16 sources are copied straight into the slot.  Small tensors are
 * gathered into one copy (Sec. 6, tensor merging).  On return all work is enqueued (a
 * load of more than tidal_config.chunks_ahead chunks paces the first part of it inside the call); completion of
 * compute_stream implies completion of the whole call.  If an adapter is
 * attached, the sources must cover every slot it touches (then the template is pristine
 * again and nothing is attached), else TIDAL_E_STATE.  A slot may appear at most once. */
int tidal_materialize(tidal_template* t, const tidal_src* srcs /* [host] */, int32_t n_src,
                      void* copy_stream, void* compute_stream);

/* The copy plan tidal_materialize would execute for these sources, without executing it
 * (host-only).  Writes at most cap pieces; returns the number of pieces of the full plan,
 * or a negative tidal_status.  assume_pinned: 1 = treat sources as pinned host memory,
 * 0 = as pageable, -1 = ask the HIP runtime (needs a GPU). */
int32_t tidal_materialize_plan(tidal_template* t, const tidal_src* srcs /* [host] */, int32_t n_src,
                               int32_t assume_pinned, tidal_copy_piece* out /* [host] out */,
                               int32_t cap);

/* Dynamic initialisation (Sec. 5.2): upload A and B of every target (converted to bf16 like
 * any weight), then update every targeted slot in place in one pass,
 *     W[i][j] <- bf16( f32(W[i][j]) + (alpha/r) * sum_k f32(B[i][k]) * f32(A[k][j]) ),
 * fp32 accumulation, one rounding.  Slots not named are not written.  TIDAL_E_STATE if an
 * adapter is already attached or a target slot was never materialised; TIDAL_E_INVAL for
 * r < 0, r > max_rank, duplicate or out-of-range slots; TIDAL_E_NOMEM if the packed adapter
 * exceeds max_adapter_bytes. */
int tidal_lora_attach(tidal_template* t, const tidal_lora_target* targets /* [host] */,
                      int32_t n_targets, void* stream);

/* Keep-alive path (Sec. 5.2): replace the attached adapter.  Bit-identical to
 * tidal_lora_detach followed by tidal_lora_attach (two roundings: W is rounded to bf16
 * after the old delta is subtracted), but a slot targeted by both adapters is read and
 * written once.  Target sets and ranks of old and new may differ. */
int tidal_lora_swap(tidal_template* t, const tidal_lora_target* targets_new /* [host] */,
                    int32_t n_targets, void* stream);

/* Cold start of a function whose adapter is known while its weights stream in:
 * tidal_materialize and tidal_lora_attach in one pass.  The dynamic part of initialisation
 * (Sec. 5.2, adaptive template state reusing) is folded into the load: every targeted slot is
 * written once, straight from the staged fp32 / fp16 source,
 *     slot[i][j] = bf16( f32(src[i][j]) + (alpha/r) * sum_k f32(B[i][k]) * f32(A[k][j]) ),
 * ONE rounding from the host-precision source (convert-then-attach rounds twice) and no
 * separate read-modify-write pass; a bf16 source is exact in its slot already and is merged in
 * place after its copy (the same single rounding).  Slots not targeted are converted as by
 * tidal_materialize.  Afterwards the adapter counts as attached (swap / detach work as after
 * tidal_lora_attach; detach leaves the slot within the merge-unmerge bound of bf16(src)).
 * Every active target's slot must be among the sources (TIDAL_E_INVAL); if an adapter is
 * already attached the sources must cover all its slots (TIDAL_E_STATE otherwise).  Other
 * errors as for the two calls.  The factors are uploaded on compute_stream first. */
int tidal_materialize_attach(tidal_template* t, const tidal_src* srcs /* [host] */, int32_t n_src,
                             const tidal_lora_target* targets /* [host] */, int32_t n_targets,
                             void* copy_stream, void* compute_stream);

/* How a LoRA pass (attach: r_old = 0; detach: r_new = 0; swap: both; fork != 0: tidal_fork_apply)
 * over n_targets slots of out x in would be launched: kernel and compile-time variant, 32-row
 * blocks a wave walks, workgroups.  Host-only introspection, like tidal_materialize_plan: tests
 * use it to show that they exercise the launch geometry the full-size workloads run with. */
typedef struct {
    char kernel[64];             /* e.g. "lora_mfma_kernel<8,0,4,inplace,pair>" (strip width / 32, padded
                                    old and new rank / 16, destination, delta tiles two at a time or all) */
    int32_t launches;            /* groups of more than 128 slots are cut into equal launches         */
    int32_t targets_per_launch;
    int32_t rank_padded_old, rank_padded_new;   /* 0, 16, 32 or 64                                    */
    int32_t blocks_per_walk;     /* 32-row blocks one wave walks down its 256-column strip             */
    int32_t waves_per_simd;      /* occupancy the variant asks for in its launch bounds                */
    int64_t workgroups;          /* of 256 threads, per launch                                         */
} tidal_lora_launch;
int tidal_lora_launch_info(const tidal_template* t, int64_t out, int64_t in, int32_t n_targets, int32_t r_old,
                           int32_t r_new, int32_t fork, tidal_lora_launch* info /* [host] out */);

/* In how many groups of targets tidal_lora_attach (swap = 0) or tidal_lora_swap (swap != 0) would
 * carry out the dynamic initialisation of Sec. 5.2 for this adapter: one group means upload, pack,
 * one pass; several mean that each group's factors cross the link while the group before it is
 * merged.  Writes the number of targets of each group, in the order given, to group_targets (at most
 * cap entries) and returns the number of groups, or a negative tidal_status (the checks of
 * tidal_lora_attach on the target list; the attach state is not looked at, a swap with nothing
 * attached is planned like an attach).  Host-only introspection, like tidal_materialize_plan: it
 * uses the link and pass rates the template has measured on its grouped calls so far (fixed
 * defaults before the first), and does not ask whether the factors are pinned (pageable factors
 * always go in one group). */
int32_t tidal_lora_upload_plan(tidal_template* t, const tidal_lora_target* targets /* [host] */,
                               int32_t n_targets, int32_t swap, int32_t* group_targets /* [host] out */,
                               int32_t cap);

/* Subtract the attached adapter's delta (same packed bf16 copy that was merged): the keep-alive
 * path of Sec. 5.2 run backwards, leaving only the static state. */
int tidal_lora_detach(tidal_template* t, void* stream);

/* Resident adapters (Sec. 5.2, adaptive template state reusing: a kept-alive function holds on to
 * dynamic state that later invocations are likely to need again, so that only what differs is loaded):
 * the packed bf16 device copy lives in caller-owned device memory, so
 * attach / swap move no host data (multi-tenant pools of adapters kept on the GPU).  A resident
 * adapter holds, per target, A transposed (in x rp) and B (out x rp), zero padded to
 * rp = 16, 32 or 64 ranks, plus A row-major (r x in) for tidal_lora_apply; the in-arena copy of
 * tidal_lora_attach / _swap holds only the first two, so this size also bounds
 * max_adapter_bytes.  tidal_adapter_required_bytes returns 0 on invalid arguments. */
size_t tidal_adapter_required_bytes(const tidal_template* t, const tidal_lora_target* targets /* [host] */,
                                    int32_t n_targets);
int tidal_adapter_upload(tidal_template* t, const tidal_lora_target* targets /* [host] */,
                         int32_t n_targets, void* dev_mem /* [device] 256-byte aligned, borrowed
                         until tidal_adapter_destroy */, size_t dev_bytes, void* stream,
                         tidal_adapter** out /* [host] out */);
int tidal_adapter_destroy(tidal_adapter* a);   /* must not be attached */
/* tidal_lora_attach / tidal_lora_swap (Sec. 5.2: the invocation's dynamic weights replace the previous
 * invocation's) with an adapter that is already on the device: the same passes over W, no host data. */
int tidal_lora_attach_adapter(tidal_template* t, const tidal_adapter* a, void* stream);
int tidal_lora_swap_adapter(tidal_template* t, const tidal_adapter* a_new, void* stream);

/* Unmerged adapters for mixed batches.  The paper's dynamic function keeps a request's LoRA
 * adapter as weights of its own next to the shared base model (Sec. 3, programming interface;
 * Sec. 5.2, adaptive template state reusing), which is what lets requests with different adapters
 * share one batch: the base projection runs once for all tokens and each request's tokens get
 *     y[t] <- bf16( y[t] + (alpha/r) * B * bf16( A * x[t] ) )         (fp32 accumulation)
 * from their own adapter.  tidal_lora_apply does that for one LoRA target slot (out x in): x is
 * n_tokens x in and y is n_tokens x out, both bf16 row-major device memory; y holds the base
 * projection's output and is updated in place.  Segment i gives tokens [token_begin, token_end)
 * to adapters[adapter] (adapter < 0, r = 0 or alpha = 0: tokens left as they are).  Segments must
 * not overlap.  Every adapter must be resident (tidal_adapter_upload on this template) and list
 * `slot` among its targets; in and out must be multiples of 8; x and y 16-byte aligned.  Nothing here
 * touches the template's weights, so it may run while an adapter is merged, and attach state is
 * not changed.  `workspace` is caller-owned device memory of at least
 * tidal_lora_apply_workspace_bytes(n_tokens) bytes, 256-byte aligned, used only during the call's
 * kernels (the rank-space intermediate bf16(A x)); calls that share a workspace must be ordered on
 * one stream.  Kernels are enqueued on `stream` after the adapters' uploads.  With
 * TIDAL_FLAG_ORDERED_ACCUM both sums run as one fused multiply-add chain in ascending index order
 * (bit-reproducible against a sequential definition, and slow). */
typedef struct tidal_lora_segment {
    int32_t adapter;       /* index into adapters[], or < 0 for "no adapter" */
    int32_t token_begin;   /* first token row of the segment                 */
    int32_t token_end;     /* one past the last token row                    */
} tidal_lora_segment;
size_t tidal_lora_apply_workspace_bytes(int32_t n_tokens);
int tidal_lora_apply(tidal_template* t, int32_t slot, const tidal_adapter* const* adapters /* [host] */,
                     int32_t n_adapters, const tidal_lora_segment* segments /* [host] */, int32_t n_segments,
                     const void* x /* [device] */, void* y /* [device] in/out */, int32_t n_tokens,
                     void* workspace /* [device] */, size_t workspace_bytes, void* stream);
/* The same for several target slots that read the same x (the query, key and value projections
 * of a layer) in one set of launches: ys[k] is the output of slots[k] (n_tokens x rows of that
 * slot).  The slots must have the same number of input columns and every adapter must target
 * all of them; the workspace must hold tidal_lora_apply_workspace_bytes(n_tokens * n_slots).
 * Results are identical to one tidal_lora_apply per slot; small batches, whose kernels are
 * bound by launch and latency rather than bandwidth, cost about the same as a single call. */
int tidal_lora_apply_multi(tidal_template* t, const int32_t* slots /* [host] */, int32_t n_slots,
                           const tidal_adapter* const* adapters /* [host] */, int32_t n_adapters,
                           const tidal_lora_segment* segments /* [host] */, int32_t n_segments,
                           const void* x /* [device] */, void* const* ys /* [host] array of [device] in/out */,
                           int32_t n_tokens, void* workspace /* [device] */, size_t workspace_bytes, void* stream);

/* For callers that cannot allocate device memory -- code under HIP graph capture, tight serving
 * loops, harnesses that forbid allocation: tidal_lora_apply for one target slot without a
 * workspace argument.  The rank-space intermediate lives in a fixed array inside the library
 * (128 bytes per token row, tidal_lora_apply_static_max_tokens() = 16384 rows, 2 MiB that each GPU
 * the library runs on holds until the process ends); the call allocates nothing, on the device or
 * through any library, and creates no HIP object.  Arguments, results and errors are those of
 * tidal_lora_apply, and the same kernels run, so the results are bit-identical to it;
 * in addition n_tokens above the maximum gives TIDAL_E_INVAL, and TIDAL_E_STATE is returned if no
 * template has done device work on the current GPU yet (uploading the adapters does).  All calls
 * on one GPU share the array, whatever template or stream they use, and it keeps the last call's
 * contents (nothing in it needs clearing: every row a call reads it has written first): calls
 * that may overlap on one GPU race and must be ordered by the caller (one stream, or events). */
int32_t tidal_lora_apply_static_max_tokens(void);
int tidal_lora_apply_static(tidal_template* t, int32_t slot, const tidal_adapter* const* adapters /* [host] */,
                            int32_t n_adapters, const tidal_lora_segment* segments /* [host] */, int32_t n_segments,
                            const void* x /* [device] */, void* y /* [device] in/out */, int32_t n_tokens,
                            void* stream);

/* Copy-on-write forks (Sec. 1: a template must stay request-agnostic, so state that an
 * invocation writes may not be shared; Sec. 5.2: a write to a forked weight goes to a new
 * tensor).  A fork owns private copies, in caller-owned device memory, of the slots an
 * invocation's adapter writes; the template's slots are only read.  tidal_fork_apply rewrites
 * every private copy from the pristine template in one pass:
 *     fork[s] <- bf16( f32(template[s]) + (alpha/r) * B * A )   for slots the adapter targets,
 *     fork[s] <- template[s]                                    for the fork's other slots
 * (a == NULL: all plain copies).  Changing adapters is just another apply: there is no unmerge,
 * so rounding never accumulates over a sequence of adapters -- the result always equals a
 * first attach bit for bit -- and the traffic is the same 4 bytes per element as the in-place
 * swap.  TIDAL_E_STATE while an adapter is merged into the template in place; TIDAL_E_INVAL if
 * the adapter targets a slot outside the fork.  Several forks of one template may coexist. */
size_t tidal_fork_required_bytes(const tidal_template* t, const int32_t* slots /* [host] */, int32_t n);
int tidal_fork_create(tidal_template* t, const int32_t* slots /* [host] copied */, int32_t n,
                      void* dev_mem /* [device] 256-byte aligned, borrowed until tidal_fork_destroy */,
                      size_t dev_bytes, tidal_fork** out /* [host] out */);
int tidal_fork_apply(tidal_fork* f, const tidal_adapter* a /* resident adapter or NULL */, void* stream);
int tidal_fork_slot_ptr(const tidal_fork* f, int32_t slot, void** dev_ptr /* [host] out */,
                        size_t* bytes /* [host] out, may be NULL */);
int tidal_fork_destroy(tidal_fork* f);

/* Device address and byte length (2*rows*cols) of a slot: where the inference kernels find the
 * weight (Sec. 4.2: the template fixes each tensor's place in device memory ahead of the load). */
int tidal_template_slot_ptr(const tidal_template* t, int32_t slot, void** dev_ptr /* [host] out */,
                            size_t* bytes /* [host] out, may be NULL */);

/* Make `stream` wait until the last tidal_materialize has filled `slot` (the
 * synchronisation events of Sec. 5.2).  Needs TIDAL_FLAG_SLOT_EVENTS; a slot that was never
 * materialised gives TIDAL_E_STATE. */
int tidal_template_slot_wait(tidal_template* t, int32_t slot, void* stream);

/* Template size rule, Eq. 1 of Sec. 5.2:  M_prefetch = max(M_model - T_TTFT * B_PCIe, 0): the
 * bytes that must already be resident so that streaming the rest hides under an inference of
 * duration T_TTFT.  Pure arithmetic, host-only; negative or non-finite inputs give 0. */
size_t tidal_prefetch_bytes(size_t model_bytes, double ttft_seconds, double link_bytes_per_second);

/* How many leading slots (in slot = access order, Sec. 4.2) fit into prefetch_bytes: the part
 * of the template to keep resident; the rest stays "memory layout only" until it is streamed in
 * by tidal_materialize at invocation time.  Host-only. */
int tidal_template_resident_prefix(const tidal_template* t, size_t prefetch_bytes,
                                   int32_t* n_slots /* [host] out */, size_t* bytes /* [host] out, may be NULL */);

/* Stand-in consumer for an inference kernel that reads a weight: adds to *dev_sum the sum of the
 * slot's bf16 bit patterns (as unsigned 16-bit integers, wrapping in 64 bits), reading the slot
 * `passes` times (passes >= 1 scales its duration; the sum grows by the same amount each pass).
 * Bandwidth-bound, enqueued on `stream`; with TIDAL_FLAG_SLOT_EVENTS it first makes `stream` wait
 * for the slot's materialisation (the injected synchronisation of Sec. 5.2).  The caller zeroes
 * *dev_sum. */
int tidal_slot_checksum(tidal_template* t, int32_t slot, int32_t passes, void* stream,
                        uint64_t* dev_sum /* [device] 8-byte aligned */);

/* Standalone conversion of n device-resident elements of `dtype` to bf16 (the kernel
 * tidal_materialize runs on each staged chunk).  src and dst 16-byte aligned, not
 * overlapping. */
int tidal_convert_device(void* dst_bf16 /* [device] */, const void* src /* [device] */, int32_t dtype,
                         int64_t n, void* stream);

/* Host->device link rate: best of `reps` timed hipMemcpyAsync of `bytes` from a pinned
 * host buffer the call allocates, into dev.  Blocks until done. */
int tidal_h2d_peak(void* dev /* [device] */, size_t bytes, int32_t reps, void* stream,
                   double* gbytes_per_s /* [host] out */);

/* What a bare in-place pass over HBM runs at in the LoRA kernels' own tiling: n matrices of
 * rows x cols 16-bit elements, back to back at dev, every 256-column strip walked down by one wave
 * in runs of blocks_per_walk blocks of 32 rows, each 16-byte word loaded, one bit flipped, stored
 * back (an even number of passes leaves the memory as it was).  4 bytes of traffic per element and
 * no arithmetic: the measured ceiling of a merge for that row pitch and walk length, next to the
 * published peak.  Best of `reps` timed passes after a warm-up one; blocks until done.  rows must
 * be a multiple of 32, cols of 256, dev 16-byte aligned and n*rows*cols*2 bytes long. */
int tidal_hbm_rmw_peak(void* dev /* [device] in/out */, int64_t rows, int64_t cols, int64_t n, int32_t blocks_per_walk,
                       int32_t reps, void* stream, double* gbytes_per_s /* [host] out */);

/* The same walk with only its loads (TIDAL_PROBE_READ) or only its stores (TIDAL_PROBE_WRITE: fills the
 * memory with an address pattern, the previous contents are lost), 2 bytes per element; TIDAL_PROBE_RMW is
 * tidal_hbm_rmw_peak.  Separates what the read side and the write side of the memory system make of a
 * row pitch and a walk length.  Arguments and errors as above; unknown mode: TIDAL_E_INVAL. */
enum { TIDAL_PROBE_RMW = 0, TIDAL_PROBE_READ = 1, TIDAL_PROBE_WRITE = 2 };
int tidal_hbm_probe(void* dev /* [device] in/out */, int64_t rows, int64_t cols, int64_t n, int32_t blocks_per_walk,
                    int32_t mode, int32_t reps, void* stream, double* gbytes_per_s /* [host] out */);

int tidal_get_stats(tidal_template* t, tidal_stats* out /* [host] out */);
int tidal_reset_stats(tidal_template* t);

/* The host-side counterpart of the per-tensor synchronisation of Sec. 5.2, for callers that want the
 * whole template rather than one slot: block until every materialisation, adapter upload, LoRA
 * attach / swap / detach and fork apply this template enqueued has completed.  tidal_lora_apply, tidal_slot_checksum and
 * tidal_convert_device only enqueue kernels on the caller's stream and complete with it. */
int tidal_template_sync(tidal_template* t);

/* End of the keep-alive period (Sec. 5.2): waits for enqueued work, then frees the handle, pinned
 * buffers and events.  Resident adapters and the arena stay with the caller. */
int tidal_template_destroy(tidal_template* t);

/* Message of the calling thread's last failed call ("" if none).  Never NULL. */
const char* tidal_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* TIDAL_H_ */
