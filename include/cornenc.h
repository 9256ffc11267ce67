/*
 * cornenc -- the encoder task and the embedding hand-off of a disaggregated
 * multimodal serving system, as a C-ABI library for one MI355X (gfx950).
 *
 * The paper splits a multimodal LLM at the encoder boundary (Sec. 2.2 "Model
 * Fission", Listing 1): an encoder task, run by its own executor on its own GPU
 * (Sec. 2.1 "Data Plane"), turns every multimodal item of a request into one
 * embedding tensor; the tensors are appended to the request in item order; the
 * LLM task, created to receive embeddings, does not run an encoder and takes the
 * tensors forwarded to it (Sec. 2.2 "Data Forwarding").  This library is the GPU
 * compute on both sides of that boundary:
 *
 *   cs_encode              the encoder task on one packed, variable-length batch
 *   cs_forward_embeddings  the consumer-side placement of received embedding rows
 *                          into the LLM's input-embedding buffer
 *
 * The paper does not describe the inside of an encoder.  Two towers are built:
 * a Qwen2.5-VL-style vision transformer (RMSNorm, 2-D/3-D rotary, window and
 * full attention, SwiGLU, 2x2 patch merger) and a Whisper-style audio encoder
 * (two k=3 convolutions, sinusoidal positions, LayerNorm, GELU MLP, pair pooling
 * and projection).
 *
 * General rules
 *  - No call throws or aborts.  Every call returns a cs_status; cs_last_error()
 *    gives a thread-local text for the last failure on the calling thread.
 *  - "dev" pointers are device memory of the current HIP device, "host" pointers
 *    are ordinary host memory.  All dev pointers must be 16-byte aligned.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  The two
 *    hot calls enqueue work on it and return; arguments are validated on the host
 *    before anything is enqueued.  cs_encode waits on the host in two cases only: a
 *    third call while the copy of the index tables of the call before the previous
 *    one has not started yet (two pinned staging slots are used in turn), and a batch
 *    whose index tables outgrow those slots (1 MiB each from create on, about 40 000
 *    tokens), which re-allocates them and so synchronises the device once.
 *  - The caller owns every buffer it passes in, the workspace included.  The library
 *    owns its repacked copy of the weights and small host staging buffers.
 *  - Threads: calls on different encoders (and the stateless calls) may run concurrently;
 *    calls on one cs_encoder must not overlap on the host (cs_encode keeps per-encoder
 *    staging state), though the work of successive calls may overlap on the GPU if they
 *    use different workspaces and streams.
 */
#ifndef CORNENC_H
#define CORNENC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  CS_OK = 0,
  CS_ERR_INVALID_ARG = 1, /* NULL pointer, misaligned pointer, bad enum, bad size   */
  CS_ERR_SHAPE = 2,       /* cu_seqlens / grid_thw inconsistent, odd grid, ...      */
  CS_ERR_WORKSPACE = 3,   /* workspace smaller than cs_encoder_query reports        */
  CS_ERR_INDEX = 4,       /* reserved for host-side index checks                    */
  CS_ERR_UNSUPPORTED = 5, /* a configuration the kernels are not built for          */
  CS_ERR_HIP = 6,         /* a HIP runtime call failed (text in cs_last_error)      */
  CS_ERR_MISSING_WEIGHT = 7,
  CS_ERR_BUSY = 8,        /* cs_channel_acquire: every slot is in use; try again later */
  CS_ERR_NO_MEMORY = 9,   /* a host allocation inside the library failed               */
  CS_ERR_TIMEOUT = 10     /* cs_xchannel_wait: nothing arrived within the time given   */
} cs_status;

typedef enum { CS_F32 = 0, CS_BF16 = 1 } cs_dtype;
/* CS_ARCH_VIT: rotary, RMSNorm, window/full attention, SwiGLU, per-patch-norm 2x2 merger (Qwen2.5-VL-style).
 * CS_ARCH_AUDIO: two convolutions, sinusoidal positions, LayerNorm, GELU MLP, pooling (Whisper-style).
 * CS_ARCH_VIT_CLS: class token, learned absolute positions, LayerNorm, full attention inside a tile,
 *   GELU MLP, a learned per-channel scale on each branch, and a projector LayerNorm(4*hidden) ->
 *   Linear -> GELU -> Linear over 2x2 patch groups (InternVL-style; the paper names that family among
 *   the models it serves, Sec. 1 and Table 1, and says nothing of its inside). */
typedef enum { CS_ARCH_VIT = 0, CS_ARCH_AUDIO = 1, CS_ARCH_VIT_CLS = 2 } cs_arch;
/* Order of an item's patch rows on input.  RASTER: (t, row, col).  MERGE_MAJOR: the order the
 * stock preprocessors of such vision towers emit, merge group by merge group: (t, row/merge,
 * col/merge, row%merge, col%merge).  The embedding rows come out in raster order of the merged
 * grid either way. */
typedef enum { CS_ORDER_RASTER = 0, CS_ORDER_MERGE_MAJOR = 1 } cs_input_order;

/* Encoder description.  Plain data; set struct_size = sizeof(cs_encoder_config). */
typedef struct {
  uint32_t struct_size;
  int32_t arch;          /* cs_arch */
  int32_t dtype;         /* cs_dtype of the weights passed to create and of `patches` */
  int32_t out_dtype;     /* cs_dtype of the embedding rows cs_encode writes          */
  int32_t patch_dim;     /* vit: 3*tp*14*14 (1176); audio: mel bins (128)            */
  int32_t hidden;        /* 1280                                                     */
  int32_t n_heads;       /* 16 (audio 20)                                            */
  int32_t head_dim;      /* 80 (audio 64); n_heads*head_dim == hidden                */
  int32_t n_layers;      /* 32, at most 64                                           */
  int32_t mlp_dim;       /* 3420 (audio 5120)                                        */
  int32_t merge;         /* vit: side of the merged patch square (2); audio: frames pooled (2) */
  int32_t merger_hidden; /* vit: width between the two merger linears (5120)         */
  int32_t out_hidden;    /* 3584                                                     */
  int32_t window;        /* vit: window side in patches (8); <= 0: every layer full  */
  uint64_t full_attn_layer_mask; /* bit l set: layer l attends over the whole item   */
  int32_t rope_sections[3];      /* rotary pairs for (t,row,col); sum == head_dim/2; audio: all 0 */
  float rope_theta;      /* 10000                                                    */
  float norm_eps;        /* 1e-6 (audio 1e-5)                                        */
  int32_t conv_kernel;   /* audio: 3                                                 */
  int32_t input_order;   /* vit: cs_input_order of the rows of `patches` inside an item */
  int32_t attn_chunk;    /* audio: tokens (frames after the stride-2 convolution) per attention chunk:
                            attention is block-diagonal over consecutive chunks of a clip, the last one
                            may be shorter; a multiple of 4; 0: the whole clip (vit: must be 0)   */
} cs_encoder_config;

/* One named weight, HOST memory, element type = config.dtype (bf16 as raw 16-bit words),
 * row-major, Linear weights as [out_features, in_features].  Names:
 *  vit:   patch_embed.weight [hidden,patch_dim]
 *         blocks.{l}.norm1.weight [hidden]          blocks.{l}.norm2.weight [hidden]
 *         blocks.{l}.attn.qkv.weight [3*hidden,hidden]  (rows: q | k | v, each head-major)  .bias
 *         blocks.{l}.attn.proj.weight [hidden,hidden]   .bias
 *         blocks.{l}.mlp.gate.weight / mlp.up.weight [mlp_dim,hidden]  .bias
 *         blocks.{l}.mlp.down.weight [hidden,mlp_dim]   .bias
 *         merger.norm.weight [hidden]
 *         merger.fc1.weight [merger_hidden, merge*merge*hidden] .bias
 *         merger.fc2.weight [out_hidden, merger_hidden]         .bias
 *  audio: conv1.weight [hidden,patch_dim,3] .bias   conv2.weight [hidden,hidden,3] .bias
 *         blocks.{l}.norm1.weight/.bias  norm2.weight/.bias
 *         blocks.{l}.attn.qkv.weight/.bias  attn.proj.weight/.bias
 *         blocks.{l}.mlp.fc1.weight [mlp_dim,hidden] .bias  mlp.fc2.weight [hidden,mlp_dim] .bias
 *         post.norm.weight/.bias   post.proj.weight [out_hidden,hidden] .bias
 *  vit_cls: patch_embed.weight [hidden,patch_dim] .bias   cls_token [hidden]
 *         pos_embed [1 + patches per tile, hidden]  (row 0: class token; row 1 + r*w + c: patch (r,c))
 *         blocks.{l}.norm1.weight/.bias  norm2.weight/.bias  attn.qkv.weight/.bias  attn.proj.weight/.bias
 *         blocks.{l}.ls1 [hidden], ls2 [hidden]   (x += ls1 * attention branch;  x += ls2 * MLP branch)
 *         blocks.{l}.mlp.fc1.weight [mlp_dim,hidden] .bias  mlp.fc2.weight [hidden,mlp_dim] .bias
 *         merger.norm.weight/.bias [4*hidden]
 *         merger.fc1.weight [merger_hidden, 4*hidden] .bias   merger.fc2.weight [out_hidden, merger_hidden] .bias
 *         (window <= 0, rope_sections all 0, merge 2, hidden <= 2048)
 * A bias that is absent from the list is taken as zero; any other absent tensor is an error. */
typedef struct {
  const char* name;
  const void* data; /* host */
  int64_t numel;
} cs_tensor;

typedef struct cs_encoder cs_encoder;

/* Builds an encoder: checks the configuration, converts and repacks the weights on the
 * host (padding, row interleaving for fused epilogues), and copies them to the current
 * device.  The caller may free `weights` afterwards.  Blocks until the copy is done. */
cs_status cs_encoder_create(const cs_encoder_config* config, const cs_tensor* weights, int32_t n_weights,
                            cs_encoder** out_encoder);

/* Frees device and host memory of the encoder.  The caller must have synchronised every
 * stream that still runs work of this encoder.  NULL is ignored. */
void cs_encoder_destroy(cs_encoder* enc);

/* Host-only: validates a batch description and reports how many embedding rows cs_encode
 * will write and how large a workspace it needs.  cu_seqlens, grid_thw as for cs_encode.
 * The plan of a batch (token permutation, attention work lists, output rows) depends only on
 * its description; the encoder keeps the plans of the last 8 distinct descriptions, so a
 * query followed by the encode, or a serving loop over a few image sizes, plans once. */
cs_status cs_encoder_query(const cs_encoder* enc, const int32_t* cu_seqlens, const int32_t* grid_thw,
                           int32_t n_items, int64_t* n_out_rows, size_t* workspace_bytes);

/* The encoder task (Sec. 2.1 "Data Plane": the executor for image, video and audio encoders;
 * Listing 1: one embedding tensor per multimodal item, in item order).
 *
 *  patches         dev  [N, patch_dim], config.dtype.  vit: the patches of all items packed
 *                       back to back, inside an item in raster order (t, row, col), inside a
 *                       patch in the order (channel, temporal, py, px).  audio: log-mel frames,
 *                       frame-major (row = frame, column = mel bin).
 *  cu_seqlens      host [n_items+1], cu_seqlens[0] = 0, item i owns rows [cu[i], cu[i+1]).
 *  grid_thw        host [n_items,3] = (t, h, w) in patches, h and w multiples of `merge`,
 *                       t*h*w == cu[i+1]-cu[i].  audio: (1, 1, frames), frames a multiple of 8 and of 2*merge.
 *                       vit_cls: an item is one tile, (1, h, w) with 1 + h*w == rows of pos_embed.
 *  out_embeddings  dev  [M, out_hidden], config.out_dtype.  vit: item i yields t*(h/2)*(w/2) rows
 *                       in raster order of the merged grid (vit_cls: (h/2)*(w/2) rows per tile, group
 *                       (R, C) = patches (2R,2C), (2R,2C+1), (2R+1,2C), (2R+1,2C+1) in that order; the
 *                       class token yields no row); audio: frames/(2*merge) rows (the stride-2 convolution, then `merge` frames pooled); items in input
 *                       order.  M = sum over items (cs_encoder_query reports it).
 *  workspace       dev, at least the size cs_encoder_query reports for this batch; contents
 *                       are scratch.  Two calls that overlap in time need two workspaces.
 *
 * Errors are reported before any work is enqueued: CS_ERR_INVALID_ARG, CS_ERR_SHAPE,
 * CS_ERR_WORKSPACE.  Results are deterministic: the same inputs give the same bits. */
cs_status cs_encode(cs_encoder* enc, const void* patches, const int32_t* cu_seqlens, const int32_t* grid_thw,
                    int32_t n_items, void* out_embeddings, void* workspace, size_t workspace_bytes,
                    void* stream);

/* cs_encode for callers that cannot allocate device memory (a tight serving loop, a harness that
 * forbids hipMalloc, code under stream capture): the same kernels and the same results, bit for bit,
 * with the workspace taken from a static array of CS_STATIC_SCRATCH_BYTES (64 MiB) that each GPU the
 * library runs on holds until the process ends.  Calls no hipMalloc / hipFree / hipHostMalloc; the
 * pinned staging slots keep the size they have.  All arguments as for cs_encode.
 *  - A batch that needs more workspace than the array holds, or index tables larger than a staging
 *    slot, is refused with CS_ERR_WORKSPACE before anything is enqueued (cs_encoder_query tells the
 *    size; the 7B-style vision tower fits about 1300 patches, one 448 x 448 image and more).
 *  - Every call on a GPU uses that GPU's one array, and the array keeps the last call's contents
 *    (every buffer in it is written before it is read, so nothing needs clearing): calls that
 *    overlap in time on one GPU race, whatever their streams and encoders; callers serialise them. */
#define CS_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
cs_status cs_encode_static(cs_encoder* enc, const void* patches, const int32_t* cu_seqlens, const int32_t* grid_thw,
                           int32_t n_items, void* out_embeddings, void* stream);

/* A recorded cs_encode, for batches small enough that the gaps between their ~330 short kernels show (one
 * to four 448 x 448 images): the launch sequence of one batch description on one set of buffers, captured
 * once into an executable HIP graph and replayed with one call.
 *  - create runs the batch once eagerly on `stream` (a stream of the caller's, not the default stream; it is
 *    synchronised), then records the same launches from that stream and instantiates the graph.  Arguments
 *    as for cs_encode.  The index tables stay in the workspace: patches, out_embeddings and the workspace
 *    belong to the graph until it is destroyed (new pixel data is written into `patches` in place; the
 *    workspace must not be used by anything else in between).  Allocates (the graph); the launches do not.
 *  - launch replays it on `stream`; results are bit-identical to cs_encode on the same inputs.
 *  - No memset node is recorded (the path clears memory with kernels only).
 * Errors: as cs_encode, plus CS_ERR_HIP if capture or instantiation fails (nothing is left behind). */
typedef struct cs_encode_graph cs_encode_graph;
cs_status cs_encode_graph_create(cs_encoder* enc, const void* patches, const int32_t* cu_seqlens,
                                 const int32_t* grid_thw, int32_t n_items, void* out_embeddings, void* workspace,
                                 size_t workspace_bytes, void* stream, cs_encode_graph** out);
cs_status cs_encode_graph_launch(cs_encode_graph* graph, void* stream);
void cs_encode_graph_destroy(cs_encode_graph* graph);

/* Host-only: how often a batch description was found in (hits) or added to (misses) the encoder's
 * plan cache since create, over cs_encoder_query, cs_encode and cs_encode_static.  Either may be NULL. */
cs_status cs_encoder_plan_cache_stats(const cs_encoder* enc, int64_t* hits, int64_t* misses);

/* The hand-off on the consumer side (Sec. 2.2 "Data Forwarding": the receiver copies the
 * forwarded tensor into its GPU memory; Listing 1: the LLM task takes embeddings instead of
 * encoding):  dst_seq[placeholder_index[i], :] = src[i, :]  as a copy of storage words.
 *
 *  src                dev [n_rows, hidden] rows of `dtype`
 *  placeholder_index  dev [n_rows] int64, flat row number in dst_seq; -1 skips the row
 *  dst_seq            dev [dst_rows, hidden]; rows not named by an index are not touched
 *  err_flag           dev int32 or NULL; set to 1 if any index is < -1 or >= dst_rows
 *                     (that row is skipped, nothing is written out of bounds); never cleared
 *                     by the library
 * hidden * sizeof(dtype) must be a multiple of 16.  Two source rows with the same index are a
 * caller error (one of them wins).  n_rows == 0 is a no-op. */
cs_status cs_forward_embeddings(const void* src, const int64_t* placeholder_index, void* dst_seq,
                                int64_t n_rows, int64_t dst_rows, int32_t hidden, int32_t dtype,
                                int32_t* err_flag, void* stream);

/* cs_channel: the hand-off as a channel between an encoder task (producer) and an LLM task
 * (consumer) that run on two streams of one process on one GPU.  In the paper a producer's tensor
 * is put into a shared buffer, the consumer is told its address, copies it into its own memory, and
 * executors wait for tensors that have not arrived yet (Sec. 2.2 "Data Forwarding", Sec. 2.1
 * "Request Lifecycle"; cost in Sec. 3 "Sidecar Overhead").  Here the shared buffer is a pool of equally sized slots in device memory, the
 * notification is the slot number with its description (rows, width, dtype), "arrived" is a HIP
 * event, and the consumer's copy is the placement itself (the scatter of cs_forward_embeddings
 * reading the slot), so rows move once and never leave HBM.  No call blocks the host:
 *
 *   producer                                   consumer
 *   cs_channel_acquire  -> slot, dev pointer
 *   cs_encode(..., out_embeddings = pointer, producer stream)
 *   cs_channel_publish(slot, rows, ...)  ----- slot number ----->  cs_channel_forward(slot, index, dst,
 *                                                                    consumer stream)
 *
 * A slot is FREE, WRITING (acquired, being produced) or READY (published, not yet forwarded).
 *  - acquire takes the lowest-numbered FREE slot and makes `producer_stream` wait until the last
 *    consumer of that slot has read it; CS_ERR_BUSY if no slot is FREE (nothing changes; call again
 *    after a forward), CS_ERR_WORKSPACE if bytes == 0 or bytes > slot_bytes.
 *  - publish records the arrival event behind everything enqueued on `producer_stream` so far, which
 *    must include all work that writes the slot; n_rows * hidden * sizeof(dtype) must not exceed the
 *    bytes reserved (CS_ERR_SHAPE); a row must be a multiple of 16 bytes (CS_ERR_UNSUPPORTED).
 *  - forward makes `consumer_stream` wait for the arrival, enqueues
 *    dst_seq[placeholder_index[i], :] = slot[i, :] exactly as cs_forward_embeddings does (same
 *    argument rules, same err_flag behaviour) and returns the slot to FREE.  A rejected call leaves
 *    the slot READY.  With n_rows == 0 nothing is enqueued.
 *  - release returns a WRITING or READY slot to FREE without placing it (a cancelled request);
 *    `stream` is the stream whose work may still touch the slot, the next producer waits for it.
 *  - describe reports a slot (any out pointer may be NULL): state, dev pointer, and for a READY slot
 *    its rows / width / dtype and whether the arrival event has completed (a host-side poll).
 * Using a slot in the wrong state is CS_ERR_INVALID_ARG.  Calls may come from different host
 * threads; they are serialised inside.  create allocates the pool (n_slots * slot_bytes rounded up
 * to 256 bytes, one hipMalloc) and two events per slot on the current device; the other calls
 * allocate nothing.  destroy must not be called while work that uses the pool is still running.
 * Producer and consumer in two processes: cs_xchannel below. */
typedef struct cs_channel cs_channel;
typedef enum { CS_SLOT_FREE = 0, CS_SLOT_WRITING = 1, CS_SLOT_READY = 2 } cs_slot_state;
#define CS_CHANNEL_MAX_SLOTS 1024
cs_status cs_channel_create(int32_t n_slots, size_t slot_bytes, cs_channel** out);
void cs_channel_destroy(cs_channel* ch);
cs_status cs_channel_acquire(cs_channel* ch, size_t bytes, void* producer_stream, int32_t* slot, void** dev_ptr);
cs_status cs_channel_publish(cs_channel* ch, int32_t slot, int64_t n_rows, int32_t hidden, int32_t dtype,
                             void* producer_stream);
cs_status cs_channel_forward(cs_channel* ch, int32_t slot, const int64_t* placeholder_index, void* dst_seq,
                             int64_t dst_rows, int32_t* err_flag, void* consumer_stream);
cs_status cs_channel_release(cs_channel* ch, int32_t slot, void* stream);
cs_status cs_channel_describe(cs_channel* ch, int32_t slot, int32_t* state, const void** dev_ptr, int64_t* n_rows,
                              int32_t* hidden, int32_t* dtype, int32_t* arrived);

/* cs_xchannel: the same hand-off between TWO PROCESSES on one GPU, as the paper's executors are
 * (separate processes joined by a per-GPU Sidecar, Sec. 2.1 "Data Plane"; the sender writes the tensor
 * to a shared buffer, notifies the receiver of its address, the receiver reads it, Sec. 2.2 "Data
 * Forwarding"; executors wait for tensors that have not arrived, Sec. 2.1 "Request Lifecycle"; the cost
 * the paper measures for this step: Sec. 3 "Sidecar Overhead").
 *
 *   producer process                                     consumer process
 *   cs_xchannel_create(name, n_slots, slot_bytes)        cs_xchannel_open(name)
 *   cs_xchannel_acquire  -> slot, dev pointer
 *   cs_encode(..., out_embeddings = pointer, stream)
 *   cs_xchannel_publish(slot, rows, ..., stream)  --->   cs_xchannel_wait(timeout) -> slot, rows, width, dtype
 *                                                        cs_xchannel_forward(slot, index, dst, stream)
 *
 * The pool of slots is device memory of the producer that the consumer maps through an IPC memory
 * handle (the pool stays under 2 GiB; rows never leave HBM).  The slot table and the notification queue
 * live in a POSIX shared-memory segment "/cornenc-<name>".  publish enqueues a host function on
 * `producer_stream` behind everything enqueued so far (which must include all work that writes the
 * slot); when that work has finished, the function marks the slot READY and queues its number: a slot
 * the consumer hears of is complete in memory.  forward enqueues the row scatter of
 * cs_forward_embeddings reading the slot (same argument rules, same err_flag behaviour) and behind it a
 * host function that hands the slot back (FREE).  No call blocks except cs_xchannel_wait, which polls
 * the queue for at most timeout_us microseconds (CS_ERR_TIMEOUT then; 0 = look once).
 *
 * Slot states: FREE -> WRITING (acquire) -> PUBLISHING (publish called) -> READY (producer's work done,
 * number queued) -> DRAINING (forward called) -> FREE (placement done).  release returns a WRITING slot
 * to FREE (a cancelled request).  A call on a slot in another state than it needs is
 * CS_ERR_INVALID_ARG and changes nothing; acquire returns CS_ERR_BUSY when no slot is FREE and
 * CS_ERR_WORKSPACE when bytes == 0 or bytes > slot_bytes; publish CS_ERR_SHAPE for more rows than were
 * reserved.  describe reports a slot (any out pointer may be NULL); t_ready_ns / t_placed_ns are
 * CLOCK_MONOTONIC readings taken when the slot last became READY / was last placed (one clock for both
 * processes, so their difference is the time the hand-off added after the producer's last kernel).
 * One producer process (any number of its threads and streams) and one consumer thread per channel.
 * create allocates (one hipMalloc, one shared segment) and open maps; the other calls allocate nothing.
 * The creator closes last: cs_xchannel_close of the creator frees the pool and removes the segment.
 * close waits for the device first (hipDeviceSynchronize), so that no host function of the closing
 * process that is still queued behind a publish or a forward refers to the channel afterwards. */
typedef struct cs_xchannel cs_xchannel;
typedef enum { CS_XSLOT_FREE = 0, CS_XSLOT_WRITING = 1, CS_XSLOT_PUBLISHING = 2, CS_XSLOT_READY = 3,
               CS_XSLOT_DRAINING = 4 } cs_xslot_state;
#define CS_XCHANNEL_MAX_SLOTS 256
cs_status cs_xchannel_create(const char* name, int32_t n_slots, size_t slot_bytes, cs_xchannel** out);
cs_status cs_xchannel_open(const char* name, cs_xchannel** out);
void cs_xchannel_close(cs_xchannel* ch);
cs_status cs_xchannel_acquire(cs_xchannel* ch, size_t bytes, int32_t* slot, void** dev_ptr);
cs_status cs_xchannel_publish(cs_xchannel* ch, int32_t slot, int64_t n_rows, int32_t hidden, int32_t dtype,
                              void* producer_stream);
cs_status cs_xchannel_wait(cs_xchannel* ch, int64_t timeout_us, int32_t* slot, int64_t* n_rows, int32_t* hidden,
                           int32_t* dtype);
cs_status cs_xchannel_forward(cs_xchannel* ch, int32_t slot, const int64_t* placeholder_index, void* dst_seq,
                              int64_t dst_rows, int32_t* err_flag, void* consumer_stream);
cs_status cs_xchannel_release(cs_xchannel* ch, int32_t slot);
cs_status cs_xchannel_describe(cs_xchannel* ch, int32_t slot, int32_t* state, const void** dev_ptr, int64_t* n_rows,
                               int32_t* hidden, int32_t* dtype, int64_t* t_ready_ns, int64_t* t_placed_ns);

/* Host-only (no GPU needed) view of the token plan cs_encode builds for a vit batch with this
 * configuration; also validates the batch description exactly as cs_encode does.
 * The towers work in an internal token order: item, frame, window (row-major over the
 * window grid), 2x2 merge group (row-major inside the window), patch inside the group.
 *  src_row   [N]   raster patch row feeding internal token i
 *  out_row   [N/4] output embedding row written by internal merged token j
 *  win_cu    [n_windows+1] internal-token boundaries of the attention windows
 * Any output pointer may be NULL.  *n_windows receives the number of windows.
 * vit_cls: a tile of h*w patches has h*w + 4 internal tokens: its patches merge group by merge group,
 * then the class token, then three padding tokens; src_row [N + 4*n_items] holds -1 for those four,
 * out_row [N/4 + n_items] holds -1 for the row they form; there are no windows (*n_windows = 0). */
cs_status cs_plan_tokens(const cs_encoder_config* config, const int32_t* cu_seqlens, const int32_t* grid_thw,
                         int32_t n_items, int32_t* src_row, int32_t* out_row, int32_t* win_cu,
                         int32_t win_cu_capacity, int32_t* n_windows);

/* Component calls: the two contraction kernels on their own, for parity tests and
 * micro-benchmarks.  All pointers dev.
 *
 * cs_linear_bf16:  C[m,n] = sum_k A[m,k] * W[n,k] + bias[n]   (bias may be NULL)
 *  A bf16 [M,lda] (lda >= K), W bf16 [N,K] with K a multiple of 64, C [M,N] of c_dtype. */
cs_status cs_linear_bf16(const void* A, int64_t lda, const void* W, const float* bias, void* C,
                         int32_t c_dtype, int64_t M, int32_t N, int32_t K, void* stream);

/* cs_attention_varlen: softmax(q k^T) v per head inside each segment; q already carries the
 * softmax scale times log2(e) (scores are exponentiated with exp2).
 *  qk   bf16 [N_tok, 2*n_heads*head_dim]  (q | k, head-major)
 *  vt   bf16 [n_heads*head_dim, ld_vt]    v transposed: vt[h*head_dim+d, token]
 *  seg_cu host int32 [n_seg+1] token boundaries, multiples of 4
 *  out  bf16 [N_tok, n_heads*head_dim]
 * head_dim 64 or 80.  Unlike the hot calls this one allocates and blocks: it builds the work list of the
 * segments on the host, uploads it with a hipMalloc and a synchronous copy, and synchronises `stream`
 * before it returns (cs_encode keeps its work lists in the plan and does neither). */
cs_status cs_attention_varlen(const void* qk, const void* vt, int64_t ld_vt, void* out, const int32_t* seg_cu,
                              int32_t n_seg, int32_t n_heads, int32_t head_dim, void* stream);

/* Timing of one step of the encoder task with HIP events on the caller's stream (measurement
 * aid; Sec. 1 mentions tracing only in passing).  After cs_encoder_time_step(enc, step), every
 * cs_encode records an event pair around each launch of that step; cs_encoder_read_timing waits
 * for the recorded events, returns the summed elapsed milliseconds and the number of launches
 * since the last read, and clears them.  step = CS_STEP_NONE switches recording off. */
typedef enum {
  CS_STEP_NONE = 0,
  CS_STEP_FRONT = 1,       /* gather/cast, rotary table, patch embed / convolutions */
  CS_STEP_NORM = 2,        /* RMSNorm / LayerNorm launches inside the blocks        */
  CS_STEP_QKV = 3,         /* QKV projection with rotary epilogue                   */
  CS_STEP_ATTN_WINDOW = 4,
  CS_STEP_ATTN_FULL = 5,
  CS_STEP_PROJ = 6,        /* attention output projection + residual                */
  CS_STEP_MLP_UP = 7,      /* gate|up with SwiGLU epilogue (audio: fc1 + GELU)      */
  CS_STEP_MLP_DOWN = 8,    /* down projection + residual                            */
  CS_STEP_BACK = 9         /* final norm, merger / pooling, output projection       */
} cs_step;
cs_status cs_encoder_time_step(cs_encoder* enc, int32_t step);
/* Host-only measurement aid: the name of the GEMM kernel instantiation (tile, waves, epilogue, tail handling,
 * MFMA shape) that `step` (CS_STEP_QKV, CS_STEP_PROJ, CS_STEP_MLP_UP or CS_STEP_MLP_DOWN) runs for a batch of
 * n_tokens tokens when it is not split over K, written as a C string to `out` (capacity >= 96). */
cs_status cs_encoder_step_kernel(const cs_encoder* enc, int32_t step, int64_t n_tokens, char* out, size_t capacity);
/* An event pair costs the stream about 5 us of idle time on either side of the launch it brackets
 * (measured: 0.36 ms per step when all 32 launches of one step are timed).  cs_encoder_time_every(enc, n)
 * times only every n-th launch of the selected step (n >= 1; default 1), counted from the call. */
cs_status cs_encoder_time_every(cs_encoder* enc, int32_t every);
cs_status cs_encoder_read_timing(cs_encoder* enc, double* total_ms, int64_t* launches);

/* cs_pack_batch: host-only choice of the items that go into the next packed cs_encode call of an
 * encoder shared by several apps (Sec. 2.2 "Component Sharing": equivalent encoder tasks share one
 * executor, so items of different requests and models queue at the same encoder).  The paper
 * names no policy; this one is first-fit in arrival order under a row budget:
 *   - pending items are given oldest first, item i with rows_i = t*h*w input rows (grid_thw as
 *     cs_encode takes it);
 *   - the oldest item is always taken, even when it alone exceeds the budget (nothing starves);
 *   - every further item, in order, is taken if it still fits (sum of rows <= row_budget) and
 *     fewer than max_items are taken; items that do not fit are skipped, later smaller ones may
 *     still be taken.
 *  selected    HOST int32 out [n_pending]: indices of the taken items, increasing
 *  n_selected  HOST out
 *  cu_seqlens  HOST int32 out [n_taken+1], may be NULL; packed_grid HOST int32 out [n_taken,3], may be
 *              NULL: the arguments of the cs_encode call over the taken items in that order
 * Errors: CS_ERR_INVALID_ARG (NULL, n_pending <= 0, max_items <= 0, row_budget <= 0), CS_ERR_SHAPE
 * (an item with a non-positive dimension, or more than 2^28 rows in the batch). */
cs_status cs_pack_batch(const int32_t* grid_thw, int32_t n_pending, int64_t row_budget, int32_t max_items,
                        int32_t* selected, int32_t* n_selected, int32_t* cu_seqlens, int32_t* packed_grid);

/* cs_patchify: pixels -> the patch rows cs_encode takes, for callers that hold decoded frames
 * (the step in front of the encoder task; the paper says nothing of preprocessing: in Listing 1 the
 * encoder task is handed the request's multimodal data as it is).  No resizing: sides must already be multiples of the patch size.
 *  frames      dev, items back to back, item i = [F_i, 3, H_i, W_i] of in_dtype (CS_F32 or CS_BF16),
 *              16-byte aligned; every item must start 16-byte aligned (it does when H*W is a multiple of 8)
 *  frame_dims  HOST int32 [n_items,3] = (F, H, W) in pixels; H, W multiples of patch; F == 1 or a
 *              multiple of temporal_patch (a single frame is shown temporal_patch times)
 *  patches     dev [N, 3*temporal_patch*patch*patch] of out_dtype: rows in raster order (t, row, col)
 *              per item, items in order; inside a row the order is (channel, frame in the temporal
 *              patch, py, px).  Values are copied (fp32 -> bf16 rounds to nearest even).
 *  grid_thw    HOST int32 [n_items,3] out, may be NULL: (t, h, w) in patches, as cs_encode takes it
 *  cu_seqlens  HOST int32 [n_items+1] out, may be NULL
 * Enqueues one kernel per 32 items on `stream`; allocates nothing.  patch must be even.
 * Errors (nothing enqueued): CS_ERR_INVALID_ARG, CS_ERR_SHAPE. */
cs_status cs_patchify(const void* frames, int32_t in_dtype, const int32_t* frame_dims, int32_t n_items,
                      int32_t temporal_patch, int32_t patch, void* patches, int32_t out_dtype,
                      int32_t* grid_thw, int32_t* cu_seqlens, void* stream);

/* Measurement aid: the rate of a bare v_mfma_f32_32x32x16_bf16 loop (no memory traffic) on the
 * current device, the ceiling the GEMMs' roofline fraction is read against.  Runs one warm-up and
 * one timed launch of 256 workgroups x 8 waves x iters x 32 MFMAs on `stream`, waits for it, and
 * writes TFLOP/s to *tflops (host).  random_operands = 0: all operands zero (nominal clock);
 * otherwise pseudo-random operands in [-1, 1], with which the board runs into its power limit.
 *  scratch  dev, at least 512 KiB (the accumulators are stored there so the loop is not removed).
 * Errors: CS_ERR_INVALID_ARG for NULL / small scratch or iters <= 0; CS_ERR_HIP from the runtime. */
cs_status cs_mfma_ceiling(void* scratch, size_t scratch_bytes, int32_t random_operands, int32_t iters,
                          double* tflops, void* stream);

const char* cs_status_string(cs_status s);
const char* cs_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* CORNENC_H */
