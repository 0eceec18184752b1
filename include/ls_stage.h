/*
 * ls_stage.h -- C ABI of the execute-while-load pipeline-stage executor (MI355X / gfx950).
 *
 * One ls_stage is one stage of an execution pipeline in the sense of the paper's
 * Section 4.1: it holds a contiguous span [layer_lo, layer_hi) of a decoder's model
 * blocks, takes the previous stage's intermediate result (or token ids, if it is the
 * first stage), produces its own intermediate result (or next-token ids, if it is the
 * last stage) and keeps its own KV cache, which never leaves the stage.  The model
 * arrives as packed blocks (Section 5, "tensor packing": one contiguous region per
 * block; "GPU memory pre-allocation": all block and intermediate buffers are sized once),
 * and a layer may run as soon as its own block has landed in device memory
 * (execute-while-load: Sections 1, 3 and 7.3), whatever has or has not arrived of the
 * later layers.  The per-layer arithmetic is the Llama-2 pre-norm decoder block that the
 * paper's Section 6 takes over from Meta's Llama inference code:
 *
 *     y = RMSNorm(x; g_attn)          q,k,v = y Wqkv^T        RoPE(q), RoPE(k)
 *     append k,v to the cache         o = causal softmax(q k^T / sqrt(hd)) v   (GQA)
 *     x += o Wo^T                     y = RMSNorm(x; g_ffn)
 *     x += (silu(y Wg^T) * (y Wu^T)) Wd^T
 *
 * Conventions
 *   - "device" pointers are HIP device memory owned by the caller; "host" pointers are
 *     ordinary host memory unless "pinned" is stated.  The library never frees or
 *     reallocates a caller buffer.  After ls_stage_create it allocates no device memory.
 *   - hip_stream arguments are a hipStream_t passed as void* (NULL = the null stream).
 *   - Every call only enqueues work; none waits for the GPU.
 *   - Every function returns LS_OK (0) or a negative ls_status.  An error that can be
 *     seen from the host arguments is reported before anything is enqueued, so a failing
 *     call has no device side effects.  ls_last_error() gives a thread-local message.
 *   - Matrices are row-major [out, in].  Activations are row-major [rows, hidden].
 *   - dtype 0 = IEEE fp32, 1 = bfloat16 (16-bit patterns, round-to-nearest-even).
 */
#ifndef LS_STAGE_H
#define LS_STAGE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LS_ABI_VERSION 1u
#define LS_DTYPE_F32 0u
#define LS_DTYPE_BF16 1u

/* Block index of the embedding table; the head block has index n_layers_total. */
#define LS_BLOCK_EMBED (-1)

typedef struct ls_stage ls_stage; /* opaque */

typedef enum {
  LS_OK = 0,
  LS_ERR_INVALID_ARG = -1,    /* null pointer, bad size, unsupported shape             */
  LS_ERR_BLOCK_RANGE = -2,    /* block index is not one this stage holds               */
  LS_ERR_NOT_LOADED = -3,     /* a block the call needs has not been enqueued for load */
  LS_ERR_ALREADY_LOADED = -4, /* block was already enqueued since the last reset       */
  LS_ERR_KV_OVERFLOW = -5,    /* a sequence would outgrow max_seq                      */
  LS_ERR_OOM = -6,            /* a caller buffer is smaller than the sizing query says */
  LS_ERR_HIP = -7             /* a HIP runtime call failed; see ls_last_error()        */
} ls_status;

/* Shape of the decoder and the limits all buffers are sized for. */
typedef struct {
  uint32_t abi_version;    /* LS_ABI_VERSION                                          */
  uint32_t dtype;          /* storage type of weights, hidden states and KV cache     */
  uint32_t n_layers_total; /* layers of the whole model (the stage holds a sub-span)  */
  uint32_t hidden;         /* d                                                       */
  uint32_t n_q_heads;      /* Hq                                                      */
  uint32_t n_kv_heads;     /* Hkv, divides Hq; query head h reads kv head h/(Hq/Hkv)  */
  uint32_t head_dim;       /* hd, even; 64 or 128 for the bf16 fast kernels           */
  uint32_t ffn;            /* F                                                       */
  uint32_t vocab;          /* V; 0 = the model has no embedding and no LM head block  */
  float rms_eps;           /* added to the mean of squares inside the square root     */
  float rope_base;         /* pair i of a head turns by pos * rope_base^(-2i/hd)      */
  uint32_t max_batch;      /* most sequences in one call                              */
  uint32_t max_seq;        /* most cached positions per sequence                      */
  uint32_t max_tokens;     /* most rows in one prefill call (>= max_batch)            */
} ls_cfg;

/*
 * KV cache of one stage; all three buffers are device memory owned by the caller
 * (Section 5 leaves runtime state of dynamic size to the serving engine).
 *   k, v      [layer_hi-layer_lo][max_batch][n_kv_heads][max_seq][head_dim], dtype
 *   seq_lens  [max_batch] int32: positions already cached per sequence.  Prefill sets
 *             it, decode adds one, both on the device in the course of the call.
 */
typedef struct {
  void* k;
  void* v;
  int32_t* seq_lens;
} ls_kv;

/* ---- packed block format (pure functions of the shape; no device access) ------------
 *
 * Section 5: all tensors of a block lie in one contiguous region, so a block moves with
 * one bulk copy; the layout has no effect on what is computed.  A decoder layer's block
 * holds, in this order, each tensor starting on a 256-byte boundary:
 *   0 attn_norm [d]   1 wqkv [(Hq+2Hkv)*hd, d] (query rows, then key rows, then value rows)
 *   2 wo [d, Hq*hd]   3 ffn_norm [d]   4 wgu [2F, d] (gate rows, then up rows)   5 wd [d, F]
 * block LS_BLOCK_EMBED: 0 embed [V, d].   block n_layers_total: 0 final_norm [d], 1 lm_head [V, d].
 */

/* Bytes of block `layer`; 0 if the shape or the index is invalid. */
size_t ls_block_bytes(const ls_cfg* cfg, int layer);

/* Number of tensors in block `layer` (6, 1 or 2); 0 if invalid. */
int ls_block_tensor_count(const ls_cfg* cfg, int layer);

/* Byte offset and byte size of tensor `index` inside block `layer`. */
ls_status ls_block_tensor(const ls_cfg* cfg, int layer, int index, size_t* offset, size_t* bytes);

/* ---- sizing queries (pure) -----------------------------------------------------------*/

/* Device bytes for the weight slab holding every block of the stage [lo, hi), including
 * the embedding block if lo == 0 and the head block if hi == n_layers_total (vocab > 0). */
size_t ls_stage_slab_bytes(const ls_cfg* cfg, int layer_lo, int layer_hi);

/* Device bytes for the intermediate results of one call at the cfg's limits. */
size_t ls_stage_workspace_bytes(const ls_cfg* cfg, int layer_lo, int layer_hi);

/* Device bytes of EACH of ls_kv.k and ls_kv.v. */
size_t ls_stage_kv_bytes(const ls_cfg* cfg, int layer_lo, int layer_hi);

/* ---- life cycle ----------------------------------------------------------------------*/

/*
 * Create the stage [layer_lo, layer_hi), 0 <= lo < hi <= n_layers_total, on the current
 * HIP device.  weight_slab and workspace are device buffers of at least the sizes the
 * queries above return (else LS_ERR_OOM), 256-byte aligned, owned by the caller, and must
 * outlive the stage.  The stage owns only host metadata and HIP events.  All blocks start
 * NOT LOADED.  *out is written only on success.
 */
ls_status ls_stage_create(const ls_cfg* cfg, int layer_lo, int layer_hi, void* weight_slab,
                          size_t slab_bytes, void* workspace, size_t ws_bytes, ls_stage** out);

/* Release the handle and its events.  Does not wait for enqueued work: synchronise first. */
void ls_stage_destroy(ls_stage* stage);

/* Shape, limits and layer span the stage was created with (any output pointer may be NULL). */
ls_status ls_stage_info(const ls_stage* stage, ls_cfg* cfg, int* layer_lo, int* layer_hi);

/* Packed size of block `layer` of this stage (0 if the stage does not hold it). */
size_t ls_stage_block_bytes(const ls_stage* stage, int layer);

/* ---- the loader (execute-while-load) -------------------------------------------------*/

/*
 * Enqueue the copy of one packed block from host memory into its place in the slab on
 * hip_stream (the "copy stream"), then record the block's event there.  host_ptr must hold
 * ls_stage_block_bytes(stage, layer) bytes, be pinned for the copy to be asynchronous, and
 * stay valid until the event has completed.  Blocks may arrive in any order (the paper's
 * Algorithm 1 hands sub-groups circularly shifted orders).  `layer` is a decoder layer in
 * [lo, hi), LS_BLOCK_EMBED (first stage) or n_layers_total (last stage), else
 * LS_ERR_BLOCK_RANGE.  A second load of a block without ls_stage_reset_blocks in between
 * is LS_ERR_ALREADY_LOADED.
 */
ls_status ls_stage_load_block(ls_stage* stage, const void* host_ptr, int layer, void* hip_stream);

/*
 * Coarser blocks: copy the packed blocks of decoder layers layer_first..layer_last (both in
 * [lo, hi), consecutive in the slab and in host memory at host_ptr, back to back) with ONE
 * bulk copy and gate all of them on its completion.  Same rules as ls_stage_load_block; if
 * any of the layers is already enqueued nothing is enqueued.  (Section 7.6 studies the block
 * count; one block per layer is the default granularity here.)
 */
ls_status ls_stage_load_layers(ls_stage* stage, const void* host_ptr, int layer_first, int layer_last,
                               void* hip_stream);

/* Mark `layer`'s block as loaded without copying: the caller has already placed the
 * packed bytes at ls_stage_block_device_ptr() and ordered that write before hip_stream's
 * current tail (the hot-start case of Section 5, model already in GPU memory). */
ls_status ls_stage_adopt_block(ls_stage* stage, int layer, void* hip_stream);

/* Device address of block `layer` inside the slab (NULL if the stage does not hold it). */
void* ls_stage_block_device_ptr(const ls_stage* stage, int layer);

/* Forget which blocks are loaded (all become NOT LOADED); the slab is not touched.  The
 * caller must have synchronised with every call that still uses the old blocks. */
ls_status ls_stage_reset_blocks(ls_stage* stage);

/* ---- the forward pass ----------------------------------------------------------------*/

/*
 * Prompt pass over `batch` sequences packed row after row without padding.
 *   in               device.  First stage of a model with vocab>0: int32 token ids
 *                    [total_tokens]; otherwise hidden states [total_tokens, hidden], dtype.
 *   cu_seqlens_dev   device int32 [batch+1], row offsets: sequence b owns rows
 *                    [cu[b], cu[b+1]) at positions 0..len_b-1; cu[0]=0, cu[batch]=total_tokens.
 *   cu_seqlens_host  host copy of the same array (used for validation and launch sizing).
 *   kv               this stage's cache; positions [0,len_b) of every layer are written,
 *                    seq_lens[b] = len_b for b < batch.
 *   out              device.  Last stage of a model with vocab>0: int32 next-token ids
 *                    [batch] (greedy, lowest index wins ties) taken at the last row of each
 *                    sequence; otherwise the residual stream after the stage's last layer,
 *                    [total_tokens, hidden], dtype, not normalised.
 *   logits_out       optional device fp32 [batch, vocab] (last stage only), or NULL.
 * Each layer's kernels are ordered after that layer's block event (the gate).  Every block
 * the stage holds must already have been enqueued by ls_stage_load_block (or adopted),
 * else LS_ERR_NOT_LOADED.  Errors: batch/total_tokens/len beyond the cfg limits
 * (LS_ERR_INVALID_ARG, LS_ERR_KV_OVERFLOW).
 */
ls_status ls_stage_prefill(ls_stage* stage, const void* in, const int32_t* cu_seqlens_dev,
                           const int32_t* cu_seqlens_host, int batch, int total_tokens,
                           const ls_kv* kv, void* out, float* logits_out, void* hip_stream);

/*
 * One generation step: one new row per sequence at position seq_lens[b], appended to the
 * cache; attends to positions 0..seq_lens[b].
 *   in        device: int32 [batch] token ids (first stage) or hidden [batch, hidden].
 *   max_ctx   host-side upper bound of seq_lens[b] over the batch before this step;
 *             max_ctx + 1 > max_seq is LS_ERR_KV_OVERFLOW.  (A sequence whose device-side
 *             length is already max_seq is left untouched by the kernels.)
 *   out / logits_out as in prefill with one row per sequence.
 */
ls_status ls_stage_decode(ls_stage* stage, const void* in, int batch, int max_ctx,
                          const ls_kv* kv, void* out, float* logits_out, void* hip_stream);

/*
 * Host-only validation: what ls_stage_prefill / ls_stage_decode would reject from their shape
 * arguments and the stage's own state (batch and token limits, cu_seqlens well-formed, every
 * block enqueued for load), without touching the device.  ls_pipeline_run calls these for
 * every (stage, micro-batch) before it enqueues anything (Section 4.3: a batch passes through
 * every stage of its pipeline, so a pass is all-or-nothing).
 */
ls_status ls_stage_check_prefill(const ls_stage* stage, const int32_t* cu_seqlens_host, int batch, int total_tokens);
ls_status ls_stage_check_decode(const ls_stage* stage, int batch, int max_ctx);

/*
 * ls_stage_decode for callers that cannot allocate and want no partial results in memory
 * they manage: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, same kernels and bit-identical results; the one difference is
 * where the decode GEMMs that split K across workgroups (batches of 17..64 rows) stage their
 * fp32 partial tiles: in a static device array of LS_STATIC_SCRATCH_BYTES inside the library
 * (one copy per GPU, held until the process ends) instead of the caller's workspace.  The
 * call allocates and frees nothing.  A step whose largest GEMM needs more than the array
 * holds (rows x columns x K-splits across workgroups x 4 bytes; 16 MiB covers 64 rows of the
 * 13B- and 70B-shaped layers, 32 rows of the 7B-shaped ones and a 32000-entry head, which
 * needs none) is LS_ERR_OOM and enqueues nothing; the stage
 * must have been created on the device that is current at the call (LS_ERR_INVALID_ARG).
 * All calls on one GPU share that GPU's array: calls that may overlap on the device (two
 * streams, two stages) race and must be ordered by the caller.  Nothing in the array has to
 * be zero at entry and its contents after the call are unspecified.
 */
#define LS_STATIC_SCRATCH_BYTES (16u << 20)
ls_status ls_stage_decode_static(ls_stage* stage, const void* in, int batch, int max_ctx,
                                 const ls_kv* kv, void* out, float* logits_out, void* hip_stream);

/* ---- measurement ---------------------------------------------------------------------*/

/* With profiling on, ls_stage_load_block brackets each copy and ls_stage_prefill brackets
 * each layer with HIP events (default off). */
ls_status ls_stage_set_profiling(ls_stage* stage, int on);

/*
 * After the caller has synchronised: per decoder layer of the stage (n <= hi-lo entries),
 * copy_ms[i]    = duration of layer lo+i's last block copy,
 * compute_ms[i] = duration of layer lo+i's kernels in the last prefill call,
 * copy_end_ms[i] / compute_end_ms[i] = completion times relative to the first recorded
 * event of the last load / prefill sequence (either pair may be NULL).
 * LS_ERR_INVALID_ARG if profiling was off or nothing was recorded.
 */
ls_status ls_stage_layer_times(ls_stage* stage, float* copy_ms, float* compute_ms,
                               float* copy_end_ms, float* compute_end_ms, int n);

/* After the caller has synchronised: duration of block `layer`'s last copy (any block the stage
 * holds, the embedding and head blocks included) and its completion time relative to the
 * start of the first copy made with profiling on since the last reset (either may be NULL). */
ls_status ls_stage_block_times(ls_stage* stage, int layer, float* copy_ms, float* copy_end_ms);

/* After the caller has synchronised: of the last prompt pass made with profiling on, the time
 * before its first decoder layer started (row maps, embedding gather or input conversion),
 * the time after its last decoder layer ended (final norm, LM head, argmax or output
 * conversion) and the whole pass (any pointer may be NULL). */
ls_status ls_stage_pass_times(ls_stage* stage, float* before_layers_ms, float* after_layers_ms, float* total_ms);

/* Operators of one decoder layer that ls_stage_probe can time. */
#define LS_OP_NONE 0
#define LS_OP_NORM 1        /* attention RMSNorm                    */
#define LS_OP_GEMM_QKV 2    /* y Wqkv^T                             */
#define LS_OP_ATTENTION 4   /* RoPE + KV append + causal attention  */
#define LS_OP_GEMM_O 5      /* x += o Wo^T                          */
#define LS_OP_GEMM_GATEUP 6 /* silu(y Wg^T) * (y Wu^T)              */
#define LS_OP_GEMM_DOWN 7   /* x += h Wd^T                          */

/*
 * Bracket every launch of operator `op` in decoder layer `layer` with a HIP event pair on
 * the call's own stream, in prefill calls (phase 0) or decode calls (phase 1); op
 * LS_OP_NONE switches the probe off and keeps what was recorded; setting an operator starts a new
 * record.  The last 512 launches are kept.  Used to measure one
 * kernel's duration inside a timed run without a profiler attached.
 */
ls_status ls_stage_probe(ls_stage* stage, int op, int layer, int phase);

/* After the caller has synchronised: durations in ms of the probed launches since the
 * probe was set, oldest first, at most `cap`; *n receives the count.  Where the operator is
 * one kernel that the library launches with the runtime's per-kernel start/stop events (the
 * bf16 GEMMs of up to 16 rows and of more than 64 rows), a duration is that kernel's own
 * start-to-stop time, as a profiler's kernel trace reports it; otherwise it is the span
 * between two events recorded around the operator's launches, which includes launch gaps. */
ls_status ls_stage_probe_times(ls_stage* stage, float* ms, int cap, int* n);

/* ---- execution pipeline over several stages (2D pipelining) ---------------------------
 *
 * Section 4.3, "2D execution pipelines" (Fig. 6a): the stages of one model form a pipeline;
 * each stage works on a different batch of requests, hands its intermediate result to the
 * next stage and starts on the next batch.  Here the stages are ls_stage handles whose
 * spans follow each other ([0,a), [a,b), ...), each driven on its own HIP stream; a batch in
 * flight is a "micro-batch".  Stage s starts micro-batch m once stage s-1 has finished m
 * (an event wait on the GPU, no host wait) and, by stream order, once it has finished
 * m-1 itself.  On one GPU the stages share the device, so this reproduces the dataflow and
 * its ordering, not the cluster's throughput.
 */
typedef struct ls_pipeline ls_pipeline; /* opaque */

/* One micro-batch on its way through the pipeline.  All pointers except cu_seqlens_host,
 * kv and handoff themselves are device memory owned by the caller. */
typedef struct {
  const void* in;                 /* input of the first stage: token ids or hidden states  */
  const int32_t* cu_seqlens_dev;  /* prompt pass only: as in ls_stage_prefill              */
  const int32_t* cu_seqlens_host; /* prompt pass only: host copy                           */
  int32_t batch;                  /* sequences in this micro-batch                         */
  int32_t total_tokens;           /* prompt pass: rows; generation step: ignored           */
  int32_t max_ctx;                /* generation step only: as in ls_stage_decode           */
  const ls_kv* kv;                /* host array [n_stages]: this micro-batch's cache in
                                     every stage (caches are per stage and per batch)      */
  void* const* handoff;           /* host array [n_stages-1]: device buffers that carry the
                                     intermediate result from stage s to s+1, each at least
                                     rows * hidden elements of dtype                       */
  void* out;                      /* output of the last stage, as in ls_stage_prefill      */
  float* logits_out;              /* optional, last stage with an LM head only             */
} ls_microbatch;

/* Build a pipeline from n_stages >= 1 stages of the same model whose layer spans are
 * consecutive (stage i ends where stage i+1 begins), else LS_ERR_INVALID_ARG.  The
 * pipeline borrows the stage handles; they must outlive it.  No GPU work. */
ls_status ls_pipeline_create(ls_stage* const* stages, int n_stages, ls_pipeline** out);

/* Release the pipeline and its events (not the stages).  Synchronise first. */
void ls_pipeline_destroy(ls_pipeline* pipe);

/*
 * Enqueue one pass of n_micro micro-batches through every stage: phase 0 = prompt pass,
 * phase 1 = one generation step.  hip_streams is a host array of n_stages streams, stage s
 * runs on hip_streams[s]; they should differ for the stages to overlap.  The hand-off
 * buffer of (stage s, micro-batch m) may be reused by the next call: stage s does not
 * overwrite it before stage s+1 has consumed the previous content (event wait).  `in`, `out`
 * and the caches are not guarded across calls: reuse them only in stream order of the first
 * / last stage's stream.  Every error the host can see -- arguments, malformed cu_seqlens, a
 * stage with a block not yet enqueued for load (LS_ERR_NOT_LOADED) -- is reported before
 * anything is enqueued, for all stages and micro-batches.  Only enqueues; never waits for the GPU.
 */
ls_status ls_pipeline_run(ls_pipeline* pipe, int phase, const ls_microbatch* mbs, int n_micro,
                          void* const* hip_streams);

/* ---- planning (pure integer functions, host only, no GPU) --------------------------------
 *
 * Section 4.2: a model of n_blocks ordered blocks is multicast from k source nodes to the
 * rest of N nodes; the nodes form k sub-groups, each fed by one source.  Algorithm 1 cuts
 * the blocks into k chunks of ceil(n_blocks/k) and lets sub-group g receive the chunks in
 * circularly shifted order g, g+1, ..., so that after ceil(n_blocks/k) steps the sub-groups
 * together hold a whole model.  Section 4.3, Algorithm 2 then builds execution pipelines from
 * one node of every sub-group; the node of sub-group g runs chunk g, i.e. the stage
 * [lo, hi) of ls_plan_chunk_span.  Indices are 0-based.
 */

/* Blocks [*lo, *hi) of chunk `chunk` (0 <= chunk < k); trailing chunks may be empty. */
ls_status ls_plan_chunk_span(int n_blocks, int k, int chunk, int* lo, int* hi);

/* order[0..n_blocks): the order in which sub-group `group` (0 <= group < k) receives the
 * blocks, e.g. the order to hand them to ls_stage_load_block (Algorithm 1). */
ls_status ls_plan_kway_order(int n_blocks, int k, int group, int32_t* order);

/* sizes[0..k): nodes per sub-group when n_nodes >= k nodes are dealt out as evenly as
 * possible (the first n_nodes % k sub-groups hold one node more). */
ls_status ls_plan_subgroup_sizes(int n_nodes, int k, int32_t* sizes);

/*
 * Execution pipelines from sub-groups with sizes[i] joinable nodes each (Algorithm 2).
 * Pipeline p consists of the nodes (group_out[j], index_out[j]), pipe_start[p] <= j <
 * pipe_start[p+1], in pipeline order; *n_pipes pipelines are written.  group_out and
 * index_out hold `capacity` entries (LS_ERR_OOM if the sizes sum to more), pipe_start
 * capacity + 1.
 */
ls_status ls_plan_pipelines(const int32_t* sizes, int k, int32_t* group_out, int32_t* index_out,
                            int32_t* pipe_start, int capacity, int* n_pipes);

/* Steps a 1 -> n_nodes binomial-pipeline multicast of n_blocks blocks takes:
 * n_blocks + ceil(log2 n_nodes) - 1 (Section 4.2); LS_ERR_INVALID_ARG (negative) on bad input. */
int ls_plan_multicast_steps(int n_blocks, int n_nodes);

/*
 * One schedule of that multicast that takes exactly n_blocks + log2(n_nodes) - 1 steps, for
 * n_nodes a power of two >= 2 and node 0 holding all blocks at the start (Section 4.2 names
 * the technique and its step count; the schedule is this library's construction).  In step
 * s node u exchanges with node u XOR 2^(s mod log2 n_nodes): dest[s * n_nodes + u] is that
 * partner and block[s * n_nodes + u] the block u sends it, or both -1 if u sends nothing in
 * step s.  A node sends at most one block and receives at most one per step, never a block
 * the receiver already holds.  dest and block hold capacity_steps * n_nodes entries
 * (LS_ERR_OOM if more steps are needed); *n_steps receives the number of steps written.
 * Host arrays; LS_ERR_INVALID_ARG on bad input.
 */
ls_status ls_plan_multicast_schedule(int n_blocks, int n_nodes, int32_t* dest, int32_t* block, int capacity_steps,
                                     int* n_steps);

/*
 * Where an intermediate result of the forward pass lies inside the caller's workspace, so that
 * a test can compare single operators with a reference: after a call has completed, the
 * region holds what the stage's LAST layer left there.  Row-major, `dtype` elements, one row
 * per row of the call:
 *   LS_WS_QKV   [rows, (Hq+2Hkv)*hd]  projections y Wqkv^T; after a prompt pass the query part
 *               is rotated (RoPE) in place, the key/value parts are as projected (the rotated
 *               keys are in the cache); after a generation step all parts are as projected
 *   LS_WS_ATTN  [rows, Hq*hd]         attention output, heads side by side
 *   LS_WS_FFN   [rows, F]             silu(y Wg^T) * (y Wu^T)
 * *offset / *bytes: position and size (at the cfg's limits) inside the workspace.
 */
#define LS_WS_QKV 1
#define LS_WS_ATTN 2
#define LS_WS_FFN 3
ls_status ls_stage_workspace_region(const ls_stage* stage, int which, size_t* offset, size_t* bytes);

/* 1 if every duration ls_stage_probe_times would return now is a kernel's own start-to-stop
 * time, 0 if some are spans between recorded events (or nothing was probed). */
int ls_stage_probe_is_kernel_exact(const ls_stage* stage);

/*
 * Measurement aids, not part of the stage's path: what this GPU sustains for the two
 * resources the path is bound by (the paper defines no such operation; bench.py reports
 * fractions of the published peaks and of these).
 * ls_probe_read_gbps: streams `bytes` (>= 16, a multiple of 16 is used) of the device buffer
 *   `buf` (16-byte aligned, only read) with the 16-byte non-temporal loads of the decode
 *   kernels, `reps` times after a warm-up; returns the GB/s of the fastest repetition.
 * ls_probe_mfma_tflops: every SIMD runs `iters` x 16 independent v_mfma_f32_16x16x32_bf16 from
 *   registers, with operands that differ from lane to lane; returns the dense bf16 TFLOP/s of
 *   the fastest of `reps` repetitions.  The rate depends on how long the loop runs: the chip
 *   holds its top clock for a few hundred microseconds (`iters` of a few thousand) and settles
 *   at what its power limit allows over milliseconds (`iters` of 50000 is about 7 ms).
 * `sink` is a device pointer to at least 4 writable bytes or NULL (the kernels never write it
 * in practice; it keeps their work from being optimised away).  Both block until done and
 * return a negative value on bad arguments or a HIP error (see ls_last_error).
 */
double ls_probe_read_gbps(const void* buf, size_t bytes, int reps, void* sink, void* hip_stream);
double ls_probe_mfma_tflops(int iters, int reps, void* sink, void* hip_stream);

/* Message of the last failing call on this thread ("" if none). */
const char* ls_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* LS_STAGE_H */
