/*
 * liver.h -- C ABI of the MI355X (gfx950) online-resharding library.
 *
 * Online resharding of mixed-parallel training state, the data path of LiveR's
 * live reconfiguration (LiveR, Section 4.6 "Streaming Resharding" and Appendix
 * A.2): model weights (bf16), fp32 master weights and Adam m / v laid out for a
 * source (TP, PP, DP) world are reshaped into a target (TP', PP', DP') world.
 *
 *   liver_plan_create   metadata-only planning (Section 4.6.1, Appendix A.2.2):
 *                       every (source view, target view) pair of each logical
 *                       tensor is intersected; non-empty intersections become
 *                       copy descriptors (the paper's TransferTask), ordered
 *                       layer-major and cut into a stream of fixed-size staging
 *                       chunks (Section 4.6.2; Section 5 gives the default chunk size).
 *   liver_pack          source half of Algorithm 1 (cutting each task's slice): gather
 *                       the pieces of one chunk from the source shards into the
 *                       contiguous staging chunk (the wire format).
 *   liver_unpack        target half of Algorithm 1 (assembling the new shard):
 *                       scatter one staging chunk into the target shards, writing
 *                       straight into the pre-allocated target storage (Appendix
 *                       A.1); optionally re-derives bf16 weights from fp32.
 *   liver_reshard       the same result in one pass, source shards -> target
 *                       shards, no staging (single-GPU fused path).
 *
 * All logical ranks' buffers live in the memory of ONE GPU.  The library never
 * allocates in pack / unpack / reshard, never synchronises the host with the
 * device in them, and never writes a source buffer (the old world stays intact
 * until the caller commits: Section 4.8, failure fallback).  Extra device
 * memory is the caller's one staging chunk plus the plan's descriptor table
 * (bounded-memory guarantee, Appendix A.1, Theorem 1).
 *
 * Physical layout conventions (the paper leaves them to the training framework;
 * these are the Megatron-style ones this library implements):
 *   - logical tensors are row-major [out_features, in_features];
 *   - column-parallel linears (q/k/v, gate/up, embeddings, lm_head) are split in
 *     contiguous row blocks over TP; row-parallel linears (o, down) in contiguous
 *     column blocks; norms, position embeddings and biases of row-parallel
 *     linears are replicated over TP;
 *   - q, k, v are one fused parameter per rank, grouped per kv-head group:
 *     [q rows of group g ; k rows of g ; v rows of g] for the rank's groups in
 *     ascending order (if TP > n_kv_heads, group g is replicated on the TP/n_kv
 *     ranks g*r..g*r+r-1: rank g*r+j holds the j-th part of the group's q rows,
 *     then all of k, then all of v; k and v are read from j = 0); gated FFNs store [gate rows of the rank ; up rows of the
 *     rank] as one parameter;
 *   - a (tp, pp) rank's parameters are flattened and packed back to back in
 *     forward order (word/position embedding on the first stage; per layer ln1,
 *     qkv, o, ln2, fc1, fc2 with each bias after its weight; final norm and
 *     lm_head -- or a second copy of the tied word embedding if PP > 1 -- on the
 *     last stage); stage pp holds layers [pp*L/PP, (pp+1)*L/PP) (or, with an
 *     interleaved schedule, vpp groups of L/(PP*vpp) layers: pp, pp+PP, ...);
 *   - the flat buffer is zero-padded to N_pad, a multiple of DP*pad_multiple
 *     elements.  LIVER_PARAM_BF16 holds all N_pad elements on every DP rank;
 *     LIVER_MASTER_F32 / LIVER_ADAM_M_F32 / LIVER_ADAM_V_F32 are split evenly:
 *     DP rank d holds elements [d*S, (d+1)*S), S = N_pad/DP (distributed
 *     optimizer).  With bucket_elems > 0 this holds per bucket (see
 *     liver_layout_t): padding sits at the end of every bucket and a DP rank
 *     holds the d-th DP-th of every bucket, concatenated;
 *   - mixture-of-experts models (n_experts > 0) keep router weights in the dense
 *     buffers and the experts' FFN weights in a second set of buffers per rank
 *     (kinds 4..7), see liver_layout_t.ep;
 *   - a value that exists several times in the source world is read from the
 *     copy with the lowest coordinate (dp = 0, tp = 0, first stage); source
 *     padding is never read; target padding is written +0.
 *
 * Buffer tables: src_bufs[rank*LIVER_NUM_KINDS + kind], dst_bufs[rank*LIVER_NUM_KINDS
 * + kind] are DEVICE pointers, rank = tp + TP*(dp + DP*pp).  Entries the plan does not use
 * (liver_plan_buffer_used == 0) may be NULL.  The tables themselves are HOST
 * arrays, read before the call returns.
 *
 * Every function returns LIVER_OK (0) or a negative LIVER_E_* code and writes
 * nothing on error.  No exceptions cross this boundary.
 */
#ifndef LIVER_H
#define LIVER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct liver_plan liver_plan_t; /* opaque, owned by the library */

/* Buffer kinds.  0..3: the dense parameters of a rank.  4..7: the same four kinds for the EXPERT parameters
 * of a mixture-of-experts model (n_experts > 0), which live in buffers of their own because they are
 * replicated and optimizer-sharded over a different group of ranks (see liver_layout_t.ep). */
enum { LIVER_PARAM_BF16 = 0, LIVER_MASTER_F32 = 1, LIVER_ADAM_M_F32 = 2, LIVER_ADAM_V_F32 = 3,
       LIVER_EXPERT_PARAM_BF16 = 4, LIVER_EXPERT_MASTER_F32 = 5, LIVER_EXPERT_ADAM_M_F32 = 6,
       LIVER_EXPERT_ADAM_V_F32 = 7, LIVER_NUM_KINDS = 8 };

/* liver_model_spec_t.flags */
enum { LIVER_GLU = 1u,         /* gated FFN: gate.w + up.w (SwiGLU); else a plain 2-layer MLP */
       LIVER_NORM_BIAS = 2u,   /* LayerNorm (weight + bias); else RMSNorm (weight only) */
       LIVER_LINEAR_BIAS = 4u, /* every linear has a bias */
       LIVER_TIED_EMBED = 8u   /* no lm_head; output projection reuses embed.word */ };

/* liver_layout_t.flags (target layout only) */
enum { LIVER_DERIVE_BF16 = 1u  /* target PARAM = round-to-nearest-even bf16 of the source MASTER
                                  element with the same logical index; source PARAM is not read */ };

enum { LIVER_OK = 0, LIVER_E_INVALID_ARG = -1, LIVER_E_UNSUPPORTED = -2, LIVER_E_NOMEM = -3,
       LIVER_E_HIP = -4, LIVER_E_NO_DEVICE = -5 };

typedef struct {
    int32_t n_layers, hidden, n_q_heads, n_kv_heads, ffn, vocab;
    int32_t max_pos;   /* rows of the learned position embedding; 0 = none */
    uint32_t flags;    /* LIVER_GLU | LIVER_NORM_BIAS | LIVER_LINEAR_BIAS | LIVER_TIED_EMBED */
    int32_t n_experts; /* > 0: mixture of experts.  Every layer's FFN is a router (router.w [n_experts, hidden],
                          a dense parameter replicated over TP) plus n_experts FFNs of hidden size `ffn`, whose
                          parameters live in the expert buffers (kinds 4..7).  0 = dense model */
} liver_model_spec_t;

typedef struct {
    int32_t tp, pp, dp;
    int32_t pad_multiple;               /* flat buffers are padded to a multiple of dp*pad_multiple */
    int32_t only_tp, only_pp, only_dp;  /* target layout: -1 = every rank, else plan only the share of
                                           the ranks with this coordinate.  Source layout: -1 = every
                                           rank, else liver_pack and liver_reshard move only the pieces
                                           READ from the ranks with this coordinate; the wire layout
                                           and liver_unpack do not change, so chunks packed under
                                           different source restrictions into one staging chunk
                                           complement each other (one source GPU each, in a real
                                           system).  Zero padding is written under every restriction */
    uint32_t flags;                     /* target layout: LIVER_DERIVE_BF16.  Source layout: 0 */
    uint32_t kind_mask;                 /* target layout: bit k (0..3) set = kinds k and k+4 take part;
                                           0 = all.  Source layout: 0 */
    int32_t vpp;                        /* model chunks per pipeline stage (interleaved schedule);
                                           0 or 1 = none.  The layers are cut into pp*vpp groups and
                                           stage p holds groups p, p+pp, p+2*pp, ... in that order */
    int32_t vocab_multiple;             /* > 0: the vocabulary of embed.word / lm_head is padded, per
                                           world, to a multiple of vocab_multiple*tp rows; every rank
                                           holds padded/tp rows; rows >= vocab are written +0 in the
                                           target and never read from the source.  0 = no padding
                                           (vocab % tp must be 0) */
    int32_t pp_first, pp_last;          /* > 0: number of layers on the first / last pipeline stage; the
                                           other stages share the remaining layers evenly.  0 = even
                                           split.  Not combinable with vpp > 1 */
    int64_t bucket_elems;               /* > 0: the flat buffer is a sequence of buckets: parameters are
                                           appended in order and a bucket closes after the parameter that
                                           brings it to >= bucket_elems elements; EVERY bucket is padded
                                           to a multiple of dp*pad_multiple and split evenly over DP, and
                                           a DP rank's fp32 buffer is the concatenation of its slices.
                                           0 = one bucket */
    int32_t ep;                         /* expert-parallel size (0 or 1 = none; must divide dp and
                                           n_experts).  DP rank d has expert-parallel index d % ep and holds
                                           experts [e*E/ep, (e+1)*E/ep) of its stage, each split over TP like
                                           a dense FFN.  A rank's expert buffer lists them layer by layer,
                                           expert by expert (fc1, fc2 with their biases), under the same
                                           bucket / padding rules with dp/ep in place of dp; it is replicated
                                           (bf16) and optimizer-sharded (fp32) over the dp/ep ranks with the
                                           same index, in ascending order; the first of them is the copy
                                           that is read.  Dense buffers do not depend on ep */
} liver_layout_t;

typedef struct {
    int64_t n_chunks;            /* staging chunks in the stream = ceil(stream_bytes / chunk_bytes) */
    int64_t n_desc;              /* descriptors of the direct path */
    int64_t n_desc_pack, n_desc_unpack;
    int64_t stream_bytes;        /* bytes on the wire, all chunks */
    int64_t bytes_read;          /* source bytes the direct path reads */
    int64_t bytes_written;       /* target bytes the direct path writes (incl. zero padding) */
    int64_t pad_bytes;           /* of bytes_written: zero padding */
    int64_t table_bytes_device;  /* the plan's only device allocation */
    int32_t n_src_ranks, n_dst_ranks;
    int32_t n_src_bufs_used, n_dst_bufs_used;
} liver_plan_info_t;

/* One copy descriptor, as the planner sees it (for inspection and tests).
 * Offsets, strides and run are in ELEMENTS of the buffer they refer to; a rank of
 * -1 means the staging chunk (whose elements have the size of the source kind's
 * type and whose rows are packed tightly).  Row i of the piece is
 * src[src_off + i*src_stride .. +run) -> dst[dst_off + i*dst_stride .. +run). */
enum { LIVER_OP_COPY = 0, LIVER_OP_CAST_BF16 = 1, LIVER_OP_ZERO = 2 };
enum { LIVER_LIST_DIRECT = 0, LIVER_LIST_PACK = 1, LIVER_LIST_UNPACK = 2 };
typedef struct {
    int32_t op;                  /* LIVER_OP_*; ZERO has no source */
    int32_t chunk;               /* pack / unpack lists: chunk index; direct list: -1 */
    int32_t slot;                /* stream order: 0 = embeddings, 1 + l = layer l, L + 1 = final norm / head */
    int32_t src_rank, src_kind;  /* -1, -1: staging chunk (unpack) or none (ZERO) */
    int32_t dst_rank, dst_kind;  /* -1, -1: staging chunk (pack) */
    int32_t reserved;
    int64_t src_off, src_stride;
    int64_t dst_off, dst_stride;
    int64_t rows, run;
} liver_desc_t;

/* Plan the reshard of `spec` from world `src` to world `dst` (Section 4.6.1;
 * the planning step that opens Algorithm 1).  Touches metadata only -- no tensor data, no data pointers.
 * chunk_bytes: size of the caller's staging chunk, a multiple of 256, >= 256.
 * If a HIP device is present the descriptor tables are uploaded to the current
 * device (the plan's single device allocation, freed by liver_plan_destroy); if
 * not, the plan is host-only: it can be inspected but pack / unpack / reshard
 * return LIVER_E_NO_DEVICE.
 * Errors: INVALID_ARG (null pointer, bad chunk_bytes, non-positive dimension),
 * UNSUPPORTED (layers do not split over the stages as asked, hidden % n_q_heads, n_q_heads % n_kv_heads,
 * ffn % tp non-zero, vocab % tp non-zero without vocab_multiple, kv heads neither split (n_kv_heads % tp == 0) nor
 * replicated evenly (tp % n_kv_heads == 0 and q heads per group % (tp/n_kv_heads) == 0); only_* out of
 * range; beyond the sanity caps: 2^16 layers, heads, experts, stages or model chunks, 2^24 for any other
 * dimension, padding multiple or rank count; a chunk_bytes so small that the stream would have more than
 * 2^20 chunks, or a plan of more than 2^22 transfer tasks), NOMEM, HIP. */
int liver_plan_create(const liver_model_spec_t* spec, const liver_layout_t* src,
                      const liver_layout_t* dst, size_t chunk_bytes, liver_plan_t** out);

/* Free the plan and its device table.  NULL is allowed.  The caller must have
 * synchronised every stream that still runs a kernel of this plan. */
void liver_plan_destroy(liver_plan_t* plan);

/* What the plan costs and moves: descriptor counts, wire bytes, bytes read and written, and
 * table_bytes_device, the plan's only device allocation -- the "transfer-plan metadata" term C of the
 * bounded-memory guarantee (Appendix A.1, Table 3 and Theorem 1: extra memory <= B + C).  `out` is a
 * caller-owned struct; nothing else is touched.  INVALID_ARG on a null pointer. */
int liver_plan_info(const liver_plan_t* plan, liver_plan_info_t* out);

/* Size in bytes of buffer (side: 0 = source world, 1 = target world; rank; kind): the extent of what the
 * sharding function S(T, r, C) of Appendix A.2.1 assigns to rank r under that world's configuration, laid out
 * as this header describes (N_pad bf16 elements for PARAM kinds, N_pad/DP fp32 elements for the others; 0 for
 * the expert kinds of a dense model).  INVALID_ARG on a null pointer or an index out of range. */
int liver_plan_buffer_bytes(const liver_plan_t* plan, int side, int rank, int kind, size_t* out);

/* 1 if any descriptor reads (side 0) / writes (side 1) that buffer, 0 if not,
 * negative on a bad argument. */
int liver_plan_buffer_used(const liver_plan_t* plan, int side, int rank, int kind);

/* Number of descriptors in a list (LIVER_LIST_*), and the i-th of them. */
int64_t liver_plan_desc_count(const liver_plan_t* plan, int list);
int liver_plan_desc(const liver_plan_t* plan, int list, int64_t i, liver_desc_t* out);

/* Launch shape of the copy kernels (a tuning knob of this implementation; the paper has no counterpart).
 * A plan is immutable and may be used from several threads and streams at once, with ONE exception: this
 * call, which is meant for the time between liver_plan_create and the plan's first data call.
 * grid_blocks workgroups of 256 threads (0 = default: one per compute unit);
 * tile_order 0 = each workgroup walks one contiguous range of tiles, 1 = workgroups interleave tile by tile,
 * 2 = groups of up to 64 tiles visited in a scattered (multiplicative-permutation) order, 3 = teams: 8 or 32
 * workgroups (by launch size) share one contiguous range and interleave inside it, a team's members sitting on
 * one XCD (a launch too small for 8 teams runs as order 0); 100 + w = teams of w workgroups (2 <= w <= 1024; the
 * grid is rounded down to a multiple of w; a grid smaller than w runs as order 0); -1 = default (teams);
 * cache_hints bit 0 = non-temporal loads, bit 1 = non-temporal stores, -1 =
 * default (direct: both; pack: loads only; unpack: stores only, so that the
 * staging chunk may stay cache-resident).  Not thread-safe against concurrent
 * launches of the same plan. */
int liver_plan_set_launch(liver_plan_t* plan, int grid_blocks, int tile_order, int cache_hints);

/* Algorithm 1, source side: gather chunk `chunk` (0 <= chunk < n_chunks) from the
 * source shards into `staging` (device, >= chunk_bytes, 256 B aligned).
 * Asynchronous on `hip_stream` (a hipStream_t; NULL = the default stream).
 * Bytes of the chunk that carry no payload are left untouched. */
int liver_pack(const liver_plan_t* plan, int chunk, const void* const* src_bufs, void* staging,
               void* hip_stream);

/* Algorithm 1, target side: scatter chunk `chunk` from `staging` into the target
 * shards (with LIVER_DERIVE_BF16: also the fused fp32 -> bf16 cast into PARAM);
 * writes the zero padding that belongs to the chunk.  Chunks are independent:
 * any order, or any subset repeated, gives the same target bytes. */
int liver_unpack(const liver_plan_t* plan, int chunk, const void* staging, void* const* dst_bufs,
                 void* hip_stream);

/* The whole reshard in one pass: source shards -> target shards, plus zero
 * padding.  Equals pack + unpack over all chunks, bit for bit. */
int liver_reshard(const liver_plan_t* plan, const void* const* src_bufs, void* const* dst_bufs,
                  void* hip_stream);

/* The whole staged reshard as a pipeline (the single-GPU analogue of the pipelined
 * point-to-point transfer through fixed-size chunks of Section 5): chunk k is packed into
 * staging[k % n_staging] on stream_pack while earlier chunks are unpacked on
 * stream_unpack; events order pack(k) -> unpack(k) -> pack(k + n_staging).  Extra
 * device memory is still O(B): n_staging chunks of chunk_bytes (1 <= n_staging <=
 * 8; `staging` is a host array of device pointers).  The two streams may be the
 * same.  Returns after enqueueing; all work has completed once stream_unpack has
 * been synchronised.  Creates and destroys 2*n_staging HIP events per call (host
 * objects; no device memory is allocated).  Every chunk's buffers are validated before the
 * first kernel is enqueued, so an argument error writes nothing. */
int liver_reshard_staged(const liver_plan_t* plan, const void* const* src_bufs, void* const* dst_bufs,
                         void* const* staging, int n_staging, void* stream_pack, void* stream_unpack);

/* The staged reshard on ONE stream with half the launches: launch k runs the unpack of chunk k-1 (out of one
 * staging chunk) and the pack of chunk k (into the other) as one grid, so the tail of each kernel is covered
 * by the head of the next (the layer-by-layer receive / assemble / send-next overlap of Algorithm 1 and the
 * pipelined chunk transfer of Section 5, folded into single launches).  Chunk k goes through staging_even if k
 * is even, staging_odd if odd (device, chunk_bytes each, 256 B aligned, distinct).  n_chunks + 1 launches in
 * all; same target bytes as liver_pack + liver_unpack, bit for bit.  Chunks that need more than one pass on
 * either side, and plans with a non-default launch shape, fall back to separate launches for that step.
 * Allocates nothing, does not synchronise; every buffer is validated before the first launch. */
int liver_reshard_staged_fused(const liver_plan_t* plan, const void* const* src_bufs, void* const* dst_bufs,
                               void* staging_even, void* staging_odd, void* hip_stream);

/* For callers that cannot allocate device memory at all -- code under HIP-graph capture, tight serving
 * loops, harnesses that forbid hipMalloc: the whole staged reshard (pack and unpack of every chunk, in order,
 * on `hip_stream`) through a staging chunk that the LIBRARY holds, a fixed device array of
 * liver_static_staging_bytes() = 64 MiB that exists on every GPU from the moment the library is loaded until
 * the process ends.  The caller passes source and target tables only.  The call allocates nothing (no
 * hipMalloc / hipFree, no events), does not synchronise, and gives the same target bytes as liver_reshard and
 * as liver_pack + liver_unpack with a caller's chunk.
 * The plan must have been created with chunk_bytes <= liver_static_staging_bytes(); a larger one is refused
 * with LIVER_E_INVALID_ARG before anything is enqueued (the message names both sizes).  Other errors as for
 * liver_pack / liver_unpack; all buffers of all chunks are validated before the first launch.
 * All calls on one GPU share that GPU's array: calls that may overlap in time there (different streams or
 * threads) race on it -- serialise them.  The array keeps the previous call's bytes; nothing depends on
 * them, since every byte of a chunk that is read was written by the same chunk's pack. */
int liver_reshard_static(const liver_plan_t* plan, const void* const* src_bufs, void* const* dst_bufs,
                         void* hip_stream);
size_t liver_static_staging_bytes(void);

/* Plumbing (no counterpart in the paper): text for a LIVER_E_* code, followed by the detail of the calling
 * thread's last failure if that failure had this code.  The pointer is valid until the thread's next call. */
const char* liver_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* LIVER_H */
