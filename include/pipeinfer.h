/* pipeinfer.h -- C ABI of the MI355X speculative-verification library.
 *
 * One target-model pipeline stage of PipeInfer on one GPU: a contiguous slice of decoder
 * layers evaluated on a micro-batch of speculated tokens over a KV cache with a tree
 * attention mask, greedy token verification, KV commit/rollback, and Early Inference
 * Cancellation as a device-visible flag probed at every layer boundary.
 *
 * Conventions
 *  - Every function returns an int32_t status: PI_OK (0), PI_CANCELLED (1, not an error)
 *    or a negative PI_E_* code.  No exceptions.
 *  - "device" pointers are caller-owned GPU memory (e.g. torch tensors); "host" pointers
 *    are ordinary CPU memory.  The library never frees or keeps a caller pointer beyond
 *    the call, except the asynchronous work enqueued on the given stream, which reads and
 *    writes the buffers of that call until the stream reaches it.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Forward,
 *    verify and rollback only enqueue work and return; load/alloc/free/read-back calls
 *    are blocking.
 *  - pi_model and pi_kv own their device memory until the matching *_free.  A pi_model
 *    carries one set of activation scratch buffers: at most one forward per model may be
 *    in flight at a time (issue them on one stream, or serialise streams with events).
 *  - A forward is one persistent kernel whose workgroups synchronise with each other, so all
 *    of them must be resident at once: the library orders every forward on a device behind
 *    the previous forward on that device, whatever model and stream they belong to (an event
 *    wait enqueued on the caller's stream; no host blocking).  Forwards of two models on two
 *    streams therefore run one after the other, never side by side.  Other long kernels of
 *    the caller that hold compute units for a long time delay a forward but cannot stop it.
 *  - Process-wide state besides the handles: that per-device launch order, and one small
 *    per-device scratch buffer that the verification calls share (see pi_verify_greedy).
 *  - Tokens per weight pass: 1 .. PI_MAX_BATCH (of one run, or of up to PI_MAX_GROUPS runs
 *    sharing the pass).  All sizes are validated on the host before any
 *    launch; a shape the kernels do not support returns PI_E_SHAPE, never a launch.
 */
#ifndef PIPEINFER_H
#define PIPEINFER_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PI_OK 0
#define PI_CANCELLED 1
#define PI_E_ARG (-1)       /* NULL/invalid argument */
#define PI_E_SHAPE (-2)     /* configuration or size not supported */
#define PI_E_OOM (-3)       /* device allocation failed */
#define PI_E_SLOT_LIVE (-4) /* a speculative write targets a live canonical cell */
#define PI_E_HIP (-5)       /* HIP runtime error */
#define PI_E_STATE (-6)     /* model not fully loaded / handle misuse */
#define PI_E_FULL (-7)      /* no free cell in the window / no free sequence identifier */
#define PI_E_BUSY (-8)      /* compaction while a partition still holds a cell of the window */

#define PI_MAX_BATCH 16  /* tokens per weight pass */
#define PI_WINDOW 64     /* cells addressable by one run's mask word */

#define PI_DTYPE_F32 0
#define PI_DTYPE_BF16 1
#define PI_DTYPE_FP8_E4M3 2 /* weight matrices only: 8-bit floats, 4 exponent bits (bias 7), 3 mantissa
                             * bits, subnormals, no infinities, 0x7f/0xff = NaN (the OCP FP8 E4M3 format) */
#define PI_DTYPE_FP4_E2M1 3 /* weight matrices only: 4-bit floats, sign, 2 exponent bits (bias 1), 1 mantissa
                             * bit: 0, 0.5, 1, 1.5, 2, 3, 4, 6 and their negatives (the OCP FP4 E2M1 format);
                             * two weights per byte, the lower-numbered column in the low nibble */
#define PI_DTYPE_FP4_E2M1_B32 4 /* weight matrices only: FP4 E2M1 nibbles as above with one power-of-two scale
                                * per 32 consecutive columns of a row, stored as a byte: weight = e2m1(nibble) *
                                * 2^(scale byte - 127), scale byte in 1 .. 254 (4.25 bits per weight) */
#define PI_LOC_HOST 0
#define PI_LOC_DEVICE 1

/* Tensor kinds for pi_model_set_tensor.  Matrices are logical [out_features][in_features]
 * row-major; norm gains are [d_model] and always fp32. */
enum {
  PI_T_EMBED = 0,      /* [vocab][d_model]            */
  PI_T_ATTN_NORM = 1,  /* [d_model], per layer        */
  PI_T_WQ = 2,         /* [n_q_heads*head_dim][d]     */
  PI_T_WK = 3,         /* [n_kv_heads*head_dim][d]    */
  PI_T_WV = 4,         /* [n_kv_heads*head_dim][d]    */
  PI_T_WO = 5,         /* [d][n_q_heads*head_dim]     */
  PI_T_FFN_NORM = 6,   /* [d_model], per layer        */
  PI_T_WG = 7,         /* [ffn][d]  (gate)            */
  PI_T_WU = 8,         /* [ffn][d]  (up)              */
  PI_T_WD = 9,         /* [d][ffn]  (down)            */
  PI_T_FINAL_NORM = 10,/* [d_model]                   */
  PI_T_LM_HEAD = 11    /* [vocab][d_model]            */
};

typedef struct pi_model pi_model;
typedef struct pi_kv pi_kv;

/* Decoder shape.  The paper does not print the decoder formulas (Section "Background and
 * Motivation" names the attention module and the MLP of a Llama-2-style layer); this
 * library evaluates: pre-norm RMSNorm(eps), bias-free projections, rotary embedding on
 * adjacent pairs with base `rope_base`, softmax(QK^T/sqrt(head_dim)) with grouped-query
 * sharing, SwiGLU MLP, final RMSNorm and an untied LM head.
 * Constraints: head_dim in {32,64,128}; d_model, n_q_heads*head_dim multiples of 32;
 * n_q_heads a multiple of n_kv_heads with ratio <= 8; vocab a multiple of 16.
 * `dtype` is the storage type of the embedding table, the KV cache and (unless
 * `weight_dtype` says otherwise) the weight matrices; `max_pos` bounds RoPE positions.
 *
 * Quantised weight streaming (the paper's models are block-quantised; Sections "Experiment
 * Setup" and the memory-bandwidth argument of "Background and Motivation"): with dtype
 * PI_DTYPE_BF16 and weight_dtype PI_DTYPE_FP8_E4M3 the seven weight matrices of every layer
 * and the LM head are stored and streamed as 8-bit floats, one byte per weight, and decoded
 * inside the projection kernels: weight = e4m3(byte) * 2^weight_scale_exp2 (one power-of-two
 * scale for the whole model; -32 <= weight_scale_exp2 <= 32).  With weight_dtype
 * PI_DTYPE_FP4_E2M1 they are stored and streamed at half a byte per weight: weight =
 * e2m1(nibble) * 2^weight_scale_exp2.  With weight_dtype PI_DTYPE_FP4_E2M1_B32 every block of 32
 * consecutive columns of a matrix row has a scale of its own (weight = e2m1(nibble) * 2^(scale
 * byte - 127); weight_scale_exp2 must be 0): the block formats of the paper's model files, in a
 * layout of our own; the scale bytes travel beside the tiles and are streamed with them.
 * Everything else (activations, embedding rows, KV cache,
 * accumulation) is as in a bf16 model.  weight_dtype 0 with dtype PI_DTYPE_BF16 is read as
 * "same as dtype". */
typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
  float rms_eps, rope_base;
  int32_t dtype;   /* PI_DTYPE_F32 | PI_DTYPE_BF16 */
  int32_t max_pos; /* positions must be < max_pos */
  int32_t weight_dtype;      /* 0 or == dtype: matrices in `dtype`; PI_DTYPE_FP8_E4M3 / PI_DTYPE_FP4_E2M1 /
                              * PI_DTYPE_FP4_E2M1_B32 (bf16 models only) */
  int32_t weight_scale_exp2; /* used with the 8-bit and 4-bit formats */
} pi_model_config;

/* Create a model: allocates device storage for all weights (in the library's own tiled
 * layout), RoPE tables and activation scratch.  Weights start unset; every tensor must be
 * supplied once with pi_model_set_tensor before the first forward (PI_E_STATE otherwise).
 * Blocking. */
int32_t pi_model_load(const pi_model_config* cfg, pi_model** out);

/* Supply one tensor.  `src` holds the logical row-major tensor in `src_dtype`
 * (PI_DTYPE_F32: float; PI_DTYPE_BF16: 16-bit bf16 patterns) at `src_loc` (host or device).
 * Matrices must come in the model's dtype or in fp32 (rounded to bf16, nearest-even, for
 * a bf16 model); the matrices of a model with 8-bit or 4-bit weights must come in that format
 * (PI_DTYPE_FP8_E4M3: [out][in] bytes; PI_DTYPE_FP4_E2M1: [out][in/2] bytes;
 * PI_DTYPE_FP4_E2M1_B32: [out][in/2] code bytes followed at once by [out][ceil(in/32)] scale
 * bytes in the same buffer; the library does not quantise; the embedding table still comes in
 * bf16 or fp32);
 * gains must be fp32.  `layer` is ignored for the three global tensors.
 * The tensor is repacked into the internal layout; `src` may be reused after return.
 * Blocking. */
int32_t pi_model_set_tensor(pi_model* m, int32_t kind, int32_t layer, const void* src,
                            int32_t src_dtype, int32_t src_loc);

int32_t pi_model_free(pi_model* m);

/* Bytes of weight storage one full forward streams (all layers + LM head), for rooflines. */
int32_t pi_model_weight_bytes(const pi_model* m, int64_t* layer_bytes, int64_t* lm_head_bytes);

/* KV cache of `n_cells` cells per layer (Section "KV Cache"; cells [0, kv_len) are the
 * canonical sequence, cells >= kv_len are free for speculative runs' private writes,
 * Section "Pipelined KV Cache Multibuffering").  Zero-filled, kv_len = 0.
 * kv_dtype: PI_DTYPE_F32 or PI_DTYPE_BF16 (values rounded nearest-even when stored).
 * n_cells must be a multiple of 16.  Blocking. */
int32_t pi_kv_alloc(const pi_model* m, int32_t n_cells, int32_t kv_dtype, pi_kv** out);
int32_t pi_kv_free(pi_kv* kv);

/* Write K and V of cells [cell_begin, cell_begin+n) of one layer from caller data laid out
 * [n][n_kv_heads][head_dim] (src_dtype/src_loc as above).  Used for synthetic prefill.
 * Does not change kv_len.  Blocking. */
int32_t pi_kv_set_cells(pi_kv* kv, int32_t layer, int32_t cell_begin, int32_t n, const void* k_src,
                        const void* v_src, int32_t src_dtype, int32_t src_loc);
/* Read cells back as fp32 into host buffers [n][n_kv_heads][head_dim].  Blocking. */
int32_t pi_kv_get_cells(const pi_kv* kv, int32_t layer, int32_t cell_begin, int32_t n,
                        float* k_dst_host, float* v_dst_host);
/* Set / read the canonical length.  Blocking. */
int32_t pi_kv_set_len(pi_kv* kv, int32_t kv_len);
int32_t pi_kv_len(const pi_kv* kv, int32_t* out);
/* Raw cache image (K then V, internal layout) for whole-buffer comparisons: size query
 * with dst_host == NULL, else copy `*nbytes` bytes to the host.  Blocking. */
int32_t pi_kv_raw(const pi_kv* kv, void* dst_host, int64_t* nbytes);

/* One run's batch (the paper's run record: batch plus token -> logits map; Section
 * "Asynchronous Speculation / State tracking").  All arrays are device pointers of n entries.
 * Token i writes its K/V to cell slots[i] (must be >= kv_len and inside the window
 * [window_base, window_base+PI_WINDOW)), and attends to cells [0, prefix_len) plus window
 * cell window_base+c for every set bit c of mask[i] (tree attention mask, Section
 * "Speculative Inference / Verification"; mask[i] must include token i's own cell). */
typedef struct {
  int32_t n;
  const int32_t* tokens;    /* used iff layer_begin == 0 */
  const int32_t* positions; /* RoPE positions */
  const int32_t* slots;
  const uint64_t* mask;
  int32_t prefix_len;
  int32_t window_base;
} pi_run_desc;

/* Evaluate layers [layer_begin, layer_end) for one run (one pipeline node's share, Section
 * "Asynchronous Speculation": each node evaluates its allocated layers and passes the
 * activations on).
 *   hidden_in  [n][d_model] fp32 device: input activations, read iff layer_begin > 0.
 *   hidden_out [n][d_model] fp32 device: written iff layer_end < n_layers and not cancelled.
 *   logits_out [n][vocab]   fp32 device: written iff layer_end == n_layers and not cancelled
 *              (logits_out[i] is the distribution of the token that follows token i).
 *   cancel_flag: device-visible int32 (device memory or mapped pinned host memory), or
 *              NULL for runs that must never stop (non-speculative runs, Section "Early
 *              Inference Cancellation / Performance considerations").  It is probed before
 *              the first layer of the call and at every layer boundary; once a non-zero
 *              value is seen no further layer starts, outputs stay untouched and the run
 *              reports PI_CANCELLED.  It may only go 0 -> 1 during a run.
 *   run_status: device-visible int32[2], written by the device: [0] = PI_OK, PI_CANCELLED,
 *              PI_E_SLOT_LIVE (a slot below kv_len or outside the window: nothing was
 *              evaluated) or PI_E_ARG (a position outside [0, max_pos): likewise),
 *              [1] = layers_done = index of the first layer NOT
 *              evaluated (== layer_end on success).  K/V of layers < layers_done were
 *              written to the run's slots; clean them with pi_kv_rollback.  [0] = PI_E_HIP
 *              means a bounded wait inside the kernel ran out (workgroups wait for each
 *              other's data for at most about two seconds): the outputs and the model's
 *              scratch state are undefined after that; free the model and the cache.
 * Asynchronous: returns PI_OK after enqueueing; read run_status after synchronising. */
int32_t pi_stage_forward(pi_model* m, pi_kv* kv, const pi_run_desc* run, int32_t layer_begin,
                         int32_t layer_end, const float* hidden_in, float* hidden_out,
                         float* logits_out, const int32_t* cancel_flag, int32_t* run_status,
                         void* stream);

/* Several speculative runs in ONE weight pass (the single-node form of the paper's "Continuous
 * Asynchronous Speculation": many small speculative runs are in flight at once and each can be
 * cancelled on its own, Section "Early Inference Cancellation"; PipeInfer on a single node is
 * the outlook of Section "Future Work").  The micro-batch of `run` holds the tokens of n_groups
 * runs; runs see each other's cells only where their masks say so.
 *   group_of_token: HOST int32[run->n], run index of every token; each of 0..n_groups-1 occurs.
 *   cancel_flags:   device-visible int32[n_groups] (or NULL: never cancel), probed like
 *                   cancel_flag of pi_stage_forward.  From the boundary at which a run's word is
 *                   seen set, the K/V of its tokens is no longer written and its rows of the
 *                   outputs are unspecified; the other runs are unaffected.  When every run is
 *                   cancelled no further layer starts and the outputs stay untouched.
 *   group_status:   device int32[n_groups][2] (or NULL), written by the device: per run
 *                   {PI_OK | PI_CANCELLED | PI_E_SLOT_LIVE, layers_done}, layers_done = first
 *                   layer whose K/V the run did NOT write.  It travels with the activations
 *                   through the stages of one pass: a run whose entry says PI_CANCELLED when a
 *                   stage starts is treated as cancelled and its entry is left as it is, so
 *                   clear the entries (any value but PI_CANCELLED) before the first stage.
 * run_status is as for pi_stage_forward; its status is PI_CANCELLED only if every run was. */
#define PI_MAX_GROUPS 16
typedef struct {
  int32_t n_groups;
  const int32_t* group_of_token;
  const int32_t* cancel_flags;
  int32_t* group_status;
} pi_group_desc;
int32_t pi_stage_forward_multi(pi_model* m, pi_kv* kv, const pi_run_desc* run, const pi_group_desc* groups,
                               int32_t layer_begin, int32_t layer_end, const float* hidden_in,
                               float* hidden_out, float* logits_out, int32_t* run_status, void* stream);

/* Greedy token-tree verification (Section "Speculative Inference / Verification"; greedy
 * sampling as in Section "Experiments").  logits[i] follows tree node i; parent[i] < i is
 * node i's parent, -1 = child of the last accepted token (parent == NULL: linear chain).
 * Walk from the root with expected = root_expected: accept the lowest-index child whose
 * draft token equals expected, then expected = argmax(logits[child]) (lowest id on ties);
 * stop at the first node without a matching child.
 * Outputs (device): accepted_nodes[n] (first accepted_count entries valid, rest -1),
 * result[2] = {accepted_count, bonus_token} where bonus_token is the target's own next
 * token after the accepted path.  vocab <= 2^24.  Asynchronous.
 * All verification calls on a device share one scratch buffer (row maxima and a counter,
 * allocated on the first call on that device): issue them on one stream or order them with
 * events; two verifications running at the same time on one device race. */
int32_t pi_verify_greedy(const int32_t* draft, const int32_t* parent, int32_t n, const float* logits,
                         int32_t vocab, int32_t root_expected, int32_t* accepted_nodes,
                         int32_t* result, void* stream);

/* pi_verify_greedy for callers that cannot allocate: code running under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same results, but the scratch
 * (row maxima and the counter of finished rows, 132 bytes) lives in a 256-byte array that is part
 * of the library's device code instead of memory allocated on first use: the call allocates
 * nothing and frees nothing, on the device or through any library.  The limit is that of the
 * other verification calls: n <= PI_MAX_BATCH rows (PI_E_SHAPE beyond; vocab <= 2^24).  Every
 * call on a GPU uses that GPU's one array and two calls that overlap in time on one GPU race:
 * issue them on one stream or order them with events.  (The first call on a device looks up the
 * array's address; that is a query, not an allocation.)  Asynchronous. */
int32_t pi_verify_greedy_noalloc(const int32_t* draft, const int32_t* parent, int32_t n, const float* logits,
                                 int32_t vocab, int32_t root_expected, int32_t* accepted_nodes,
                                 int32_t* result, void* stream);

/* The same for a run that builds on another run's speculation (Section "Continuous
 * Speculation": trees build on the previous trees, so a rejected speculation takes its
 * descendants with it), decided on the device so that runs can be queued back to back:
 *   prev_result (device, may be NULL): the result[2] of the run this one builds on, written
 *     earlier on the same stream; this run counts only if that run accepted all of its
 *     prev_n tokens, and its bonus token is then the expectation for this run's root
 *     (root_expected is ignored).  NULL: root_expected is used as in pi_verify_greedy.
 *   run_status (device, may be NULL): the run_status of this run's forward; the run counts
 *     only if run_status[0] == PI_OK (a cancelled run's logits are not there).
 * A run that does not count yields accepted_nodes all -1 and result = {0, -1}.  Calls share
 * one scratch buffer: issue them on one stream.  Asynchronous. */
int32_t pi_verify_greedy_chained(const int32_t* draft, const int32_t* parent, int32_t n, const float* logits,
                                 int32_t vocab, int32_t root_expected, const int32_t* prev_result, int32_t prev_n,
                                 const int32_t* run_status, int32_t* accepted_nodes, int32_t* result, void* stream);

/* Commit / roll back a run's cells (Sections "KV Cache" and "Pipelined KV Cache
 * Multibuffering / Sequence partitions"): the cells of the accepted path are copied, all
 * layers, to canonical cells kv_len .. kv_len+a-1 in path order, every other cell in
 * slots[] is zero-filled (free again), and kv_len += a.  accepted_nodes/result are the
 * device outputs of pi_verify_greedy; pass result == NULL to discard the whole run
 * (cancelled run: a = 0).  Asynchronous; kv_len is updated on the device.
 * slots[] and the result are device data that may come from a forward the device refused
 * (PI_E_SLOT_LIVE, PI_E_ARG): only cells in [kv_len, n_cells) are read as a source or zero-filled
 * -- a slot below kv_len (a live canonical cell) or outside the cache is skipped -- and the path
 * is cut before the first accepted entry that is not a token of the run with such a cell, and at
 * n_cells.  Rolling back a refused run therefore leaves the cache exactly as it was. */
int32_t pi_kv_rollback(pi_kv* kv, const int32_t* slots, int32_t n, const int32_t* accepted_nodes,
                       const int32_t* result, void* stream);

/* ---- KV cell metadata and sequence partitions ------------------------------------------
 * Sections "KV Cache" and "Pipelined KV Cache Multibuffering": every cache cell carries the
 * position of its entry and the set of sequences it belongs to; runs are kept apart by giving
 * each a sequence identifier of its own, cache edits are edits of this metadata, and the
 * attention mask is built from it.  Sequence 0 is the canonical sequence; identifiers
 * 1 .. n_seq-1 are partitions, handed out first-in first-out.  A cell is canonical iff
 * sequence 0 is in its set, and free iff it is in no sequence.
 *
 * The table lives in device memory (pos[n_cells] int32, -1 = free; seq[n_cells] uint32, bit s
 * = sequence s) so that every edit below is a small kernel enqueued on `stream`, in order with
 * the forward, verify and rollback calls of the same stream; only the queue of free
 * identifiers is host state.  A pi_kvmeta is not tied to one pi_kv: it describes cells by
 * index.  Device arguments: positions[n] int32, tok_seq[n] uint32 (the sequences token i
 * belongs to: one bit for a linear run, one bit per branch through the node for a tree),
 * slots/masks/status words as stated.  n is 1 .. PI_MAX_BATCH.  The calls on one table share
 * its device state (and the mask builder its counters): issue them on one stream, or order
 * them with events; the host-side queue is not thread-safe.
 *
 * Token i sees cell c iff seq[c] & tok_seq[i] != 0 and pos[c] <= positions[i]. */
#define PI_MAX_SEQ 32
#define PI_SEQ_CANONICAL 0
#define PI_POS_MAX 0x7fffffff /* "no upper bound" for position ranges [p0, p1) */

typedef struct pi_kvmeta pi_kvmeta;

/* n_cells >= 1, 2 <= n_seq <= PI_MAX_SEQ.  All cells free; the queue holds 1, 2, ...,
 * n_seq-1 in this order.  Blocking. */
int32_t pi_kvmeta_alloc(int32_t n_cells, int32_t n_seq, pi_kvmeta** out);
int32_t pi_kvmeta_free(pi_kvmeta* meta);
/* Take the identifier at the head of the queue (Section "Sequence partitions").  Host only,
 * no device work.  PI_E_FULL when every partition is in use. */
int32_t pi_kvmeta_seq_acquire(pi_kvmeta* meta, int32_t* seq_out);
/* The run that held `seq` is over: the identifier leaves every cell that is not canonical
 * (cells left in no sequence are free), then joins the tail of the queue.  The device part
 * is asynchronous; an identifier acquired again is safe to use on the same stream.
 * PI_E_ARG if `seq` is not currently held. */
int32_t pi_kvmeta_seq_release(pi_kvmeta* meta, int32_t seq, void* stream);
/* Mark cells [cell_begin, cell_begin+n) as holding positions pos_begin .. in the sequences
 * of seq_mask (prefilled entries); seq_mask 0 frees them.  Asynchronous. */
int32_t pi_kvmeta_fill(pi_kvmeta* meta, int32_t cell_begin, int32_t n, int32_t pos_begin, uint32_t seq_mask,
                       void* stream);
/* Cells for a run's new entries: token i gets the i-th lowest free cell of the window
 * [window_base, window_base+PI_WINDOW), which then holds (positions[i], tok_seq[i]).
 * slots_out[n] (device) receives the cells; status[0] (device) PI_OK, or PI_E_FULL when the
 * window has fewer than n free cells, or PI_E_ARG when a token has a negative position, no
 * sequence or a sequence the table does not have: then nothing changes and slots_out is all
 * -1 (which a forward refuses with PI_E_SLOT_LIVE).  Asynchronous. */
int32_t pi_kvmeta_place(pi_kvmeta* meta, int32_t n, const int32_t* positions, const uint32_t* tok_seq,
                        int32_t window_base, int32_t* slots_out, int32_t* status, void* stream);
/* Entries of sequence `src` at positions [p0, p1) also become entries of every sequence in
 * dst_mask: a copy that moves no data (Sections "Pipelined KV Cache Multibuffering", "Early
 * cache entry sharing").  Asynchronous. */
int32_t pi_kvmeta_seq_cp(pi_kvmeta* meta, int32_t src, uint32_t dst_mask, int32_t p0, int32_t p1, void* stream);
/* Entries at positions [p0, p1) leave every sequence in seq_mask; a cell left in no sequence
 * is free (Section "KV Cache": rejected entries are removed by editing metadata).
 * Asynchronous. */
int32_t pi_kvmeta_seq_rm(pi_kvmeta* meta, uint32_t seq_mask, int32_t p0, int32_t p1, void* stream);
/* Section "Sequence acceptance and propagation": the accepted path of a run joins every
 * sequence, up to and including the position of the last accepted token and no further.
 * accepted_nodes/result are pi_verify_greedy's device outputs; the branch is the lowest
 * sequence of tok_seq[last accepted node]; result[0] == 0 changes nothing.  Asynchronous. */
int32_t pi_kvmeta_accept(pi_kvmeta* meta, int32_t n, const int32_t* positions, const uint32_t* tok_seq,
                         const int32_t* accepted_nodes, const int32_t* result, void* stream);
/* The attention mask from the metadata (Section "KV Cache"), in the form pi_run_desc takes:
 * mask_out[i] bit c = token i sees cell window_base+c (bits of cells below prefix_len stay
 * clear: the prefix covers them).  n_unexpressed[0] (device) counts the (token, cell) pairs
 * that this form gets wrong -- a cell below prefix_len the token must not see, or a visible
 * cell in neither prefix nor window; run a forward only if it is 0.  Asynchronous. */
int32_t pi_kvmeta_build_mask(pi_kvmeta* meta, int32_t n, const int32_t* positions, const uint32_t* tok_seq,
                             int32_t prefix_len, int32_t window_base, uint64_t* mask_out,
                             int32_t* n_unexpressed, void* stream);
/* Move the canonical cells of the window [prefix_len, prefix_len+PI_WINDOW) down to cells
 * prefix_len, prefix_len+1, ... in position order: metadata, and K/V of every layer of `kv`
 * (may be NULL: metadata only).  Cells moved away from and not refilled are free; their
 * data stays.  result[2] (device) = {status, dense length}: PI_E_BUSY with nothing changed
 * while a cell of the window belongs to partitions only or two canonical window cells hold
 * one position; else PI_OK, and kv's canonical length becomes the dense length.  No run may
 * be in flight on another stream.  Asynchronous. */
int32_t pi_kvmeta_compact(pi_kvmeta* meta, pi_kv* kv, int32_t prefix_len, int32_t* result, void* stream);
/* Copy the table to the host (either pointer may be NULL).  Blocking. */
int32_t pi_kvmeta_read(const pi_kvmeta* meta, int32_t* pos_host, uint32_t* seq_host);

/* ---- Head-node run bookkeeping (host only: no device work, callable without a GPU) -------
 * Sections "State tracking", "Invalidation detection", "Cancellation back-propagation" and
 * "Reactive speculation": every run in flight has a record in a FIFO queue holding its
 * speculated tokens and positions; after every sampling phase the queue is searched for runs
 * that are superfluous (highest position below the position of the last accepted token) or
 * invalidated (their tokens do not continue the accepted ones) and those are cancelled: for a
 * speculative run the scheduler stores 1 into the run's cancel word -- the word a forward of
 * that run polls at every layer boundary -- while a non-speculative run is only marked (it
 * must still be evaluated in full; just its sampling is skipped).  The confidence cutoff for
 * further speculation rises by `recovery` with every speculation issued, returns to `base`
 * when a completed run is accepted, and falls by `decay` when speculation stops for lack of
 * confidence while no logits are waiting.  Positions count tokens from 0.  Not thread-safe. */
#define PI_RUN_SUPERFLUOUS 1
#define PI_RUN_INVALIDATED 2

typedef struct pi_sched pi_sched;

int32_t pi_sched_create(double base_cutoff, double recovery, double decay, pi_sched** out);
int32_t pi_sched_free(pi_sched* s);
/* Create the record of a run that is about to start and append it to the queue.
 *   assumed[n_assumed]: tokens at positions assumed_pos0 .. that the run builds on and that
 *     were still speculation when it started (may be empty);
 *   tokens/parent/positions[n]: the run's own batch (parent -1 = root; parent < child; all
 *     roots at one position, a child one position after its parent);
 *   cancel_word: host-visible address of the run's device-visible cancel word (e.g. mapped
 *     pinned memory), or NULL; it must stay valid until pi_sched_complete_run.
 * run_id receives a unique identifier (0, 1, 2, ... in creation order). */
int32_t pi_sched_begin_run(pi_sched* s, int32_t speculative, const int32_t* assumed, int32_t n_assumed,
                           int32_t assumed_pos0, const int32_t* tokens, const int32_t* parent,
                           const int32_t* positions, int32_t n, volatile int32_t* cancel_word, int32_t* run_id);
/* A sampling phase has ended: tokens[n] join the accepted sequence; run_completed != 0 says
 * they come from a completed run (the cutoff returns to its base).  The queue is then
 * searched, oldest run first, by the position method, then the token method; every run newly
 * found is reported once in ids/reasons/signalled (capacity cap; *n_found is the number
 * found, which may exceed cap) and, if speculative, has its cancel word set. */
int32_t pi_sched_accept_tokens(pi_sched* s, const int32_t* tokens, int32_t n, int32_t run_completed, int32_t* ids,
                               int32_t* reasons, int32_t* signalled, int32_t cap, int32_t* n_found);
/* The run's result has been dealt with: its record leaves the queue; *state receives 0,
 * PI_RUN_SUPERFLUOUS or PI_RUN_INVALIDATED.  PI_E_ARG for an unknown run. */
int32_t pi_sched_complete_run(pi_sched* s, int32_t run_id, int32_t* state);
/* Reactive speculation. */
int32_t pi_sched_want_speculation(const pi_sched* s, double confidence, int32_t* yes);
int32_t pi_sched_on_speculated(pi_sched* s);
int32_t pi_sched_on_speculation_stopped(pi_sched* s, int32_t logits_waiting);
/* Read-back: the current cutoff, the number of accepted tokens, the queue (ids[cap], oldest
 * first; *n_runs is the queue length). */
int32_t pi_sched_state(const pi_sched* s, double* cutoff, int32_t* n_accepted, int32_t* ids, int32_t cap,
                       int32_t* n_runs);

/* ---- Continuous asynchronous speculation: the head node's loop ------------------------------
 * Sections "Asynchronous Speculation", "Continuous Speculation", "Pipelined KV Cache
 * Multibuffering" and "Early Inference Cancellation", with one GPU's stream in the role of the
 * pipeline: verification runs are queued back to back; while the oldest has not finished, further
 * micro-batches of draft tokens are issued, each a run with a sequence partition, a record and a
 * cancel word of its own, each building on the entries of the one before it (early sharing); when a
 * result arrives it is sampled (greedy), its accepted entries join every sequence, and every queued
 * run the new tokens contradict is cancelled through its cancel word.  The loop only sequences the
 * entry points above (pi_sched_*, pi_kvmeta_*, pi_stage_forward_multi, pi_verify_greedy_chained,
 * pi_kvmeta_compact) on one stream; the output is the token sequence plain greedy decoding gives.
 *
 * The draft model is the caller's: draft(ctx, position, &token, &confidence) returns PI_OK and the
 * draft model's token for `position` with its confidence in [0, 1] (the loop stops extending a
 * micro-batch when the confidence is below the reactive cutoff); alternative (may be NULL) returns 1
 * and the draft model's second choice for `position`, 0 if it has none, a negative status on error:
 * with it a run is a small tree, its chain plus one alternative leaf hanging at least two positions
 * above the chain's end, each branch with a partition of its own.  Both are called from inside
 * pi_spec_generate, on the calling thread; a non-zero status ends the call with that status.
 *   prefix_len: the cache holds canonical cells 0 .. prefix_len-1 (positions 0 .. prefix_len-1);
 *   first_token: the accepted token at position prefix_len, whose entry is not in the cache yet;
 *   depth: weight passes in flight (1..16); micro_batch: draft tokens per run (1..4);
 *   runs_per_pass: consecutive runs sharing one pass over the weights (1..8); n_seq: sequence
 *   identifiers of the cell metadata (2..PI_MAX_SEQ); base_cutoff/recovery/decay: as pi_sched_create.
 * The cache must have room for the window: prefix_len + PI_WINDOW <= n_cells, and as generation
 * goes on, accepted length + PI_WINDOW <= n_cells (PI_E_SHAPE otherwise); positions must stay below
 * the model's max_pos (PI_E_ARG).  A pi_spec owns its metadata table, its run records and its
 * buffers; the model and the cache stay the caller's and must not be used by others meanwhile. */
typedef struct pi_spec pi_spec;
typedef int32_t (*pi_draft_fn)(void* ctx, int32_t position, int32_t* token, double* confidence);
typedef int32_t (*pi_alternative_fn)(void* ctx, int32_t position, int32_t* token);
typedef struct {
  int32_t prefix_len, first_token;
  int32_t depth, micro_batch, runs_per_pass, n_seq;
  double base_cutoff, recovery, decay;
  pi_draft_fn draft;
  pi_alternative_fn alternative; /* may be NULL */
  void* ctx;
} pi_spec_config;
typedef struct {
  int64_t passes, runs, non_speculative, speculative, discarded, cancelled, layers_skipped, tokens_speculated,
      tokens_accepted_from_drafts, compactions, cutoff_stops, tree_runs, alternatives_accepted;
} pi_spec_stats;
/* Blocking (allocates its buffers; `stream` is the stream every later call of this pi_spec uses). */
int32_t pi_spec_create(pi_model* m, pi_kv* kv, const pi_spec_config* cfg, void* stream, pi_spec** out);
/* Run until n_tokens have been generated after first_token and copy them to tokens_out (host);
 * a later call with a larger n_tokens continues and returns the longer sequence from its start.
 * Blocking.  After an error the handle only accepts pi_spec_get_stats and pi_spec_free. */
int32_t pi_spec_generate(pi_spec* s, int32_t n_tokens, int32_t* tokens_out);
/* Wait for every pass in flight, deal with its results, and fold the window's canonical cells into
 * the dense prefix (pi_kvmeta_compact on the loop's table and the cache): afterwards cells
 * 0 .. *dense_len-1 hold positions 0 .. *dense_len-1, the cache's canonical length is *dense_len,
 * and *n_accepted tokens (prompt included) are accepted, the last of which has no entry yet
 * (*dense_len == *n_accepted - 1).  Either pointer may be NULL.  Blocking. */
int32_t pi_spec_settle(pi_spec* s, int32_t* n_accepted, int32_t* dense_len);
/* The loop's cell metadata as pi_kvmeta_read gives it (n_cells entries each; either may be NULL).
 * Blocking. */
int32_t pi_spec_read_cells(const pi_spec* s, int32_t* pos_host, uint32_t* seq_host);
int32_t pi_spec_get_stats(const pi_spec* s, pi_spec_stats* out);
int32_t pi_spec_free(pi_spec* s);

/* Device-visible address of pinned, mapped host memory (e.g. a cancel word the head node
 * stores into from the host): host_ptr must lie in memory allocated as pinned host memory.
 * PI_E_HIP if it does not. */
int32_t pi_mapped_device_pointer(void* host_ptr, void** device_ptr);

const char* pi_strerror(int32_t status);

/* Tuning hook (not needed for correct use): phase 0..4 (QKV, O, gate/up, down, LM head): ask
 * for at least `s_k` column slices in that projection phase; 0 restores the built-in choice, and
 * the library still rounds up to a split the tile count, grid and LDS allow.  phase 5: s_k != 0
 * makes later runs record the barrier timestamps pi_debug_read_trace returns (off by default:
 * reading the clock at every barrier costs time).  phase 6: s_k = KiB of LDS the staged
 * activations of every projection phase should stay under (16 .. 150; 0 restores the built-in choice):
 * a larger figure means fewer column slices and more staging per workgroup.  phase 7: s_k = weight tiles
 * (1 KiB each) a wave may ask for ahead of a phase, into LDS, while it waits for the phase to begin
 * (0 restores the built-in choice, 1 = none, otherwise an even figure up to 64; always limited by the
 * LDS the projection phases leave free).  phase 8: s_k = attention work units aimed at per 100
 * workgroups (0 restores the built-in 75; units are handed out in the order in which workgroups
 * finish the QKV projection, so below 100 the slowest take none). */
int32_t pi_debug_set_plan(pi_model* m, int32_t phase, int32_t s_k);
/* Debug hook: copy `count` floats of an activation scratch buffer of the last run to the host
 * (which: 0 residual stream x[n][d], 1 q[n][Hq*hd], 2 attention output [n][Hq*hd],
 * 3 SwiGLU output [n][ffn]).  Blocking. */
int32_t pi_debug_read_scratch(pi_model* m, int32_t which, float* dst_host, int64_t count);
/* Debug hook: device timestamps (100 MHz clock) taken by workgroup 0 each time it passes a grid
 * barrier of the last run: [0] run latch, [1] stage input ready, then two per layer (after the
 * output projection; layer boundary).  count <= 5 * n_layers + 8.  Blocking. */
int32_t pi_debug_read_trace(pi_model* m, uint64_t* dst_host, int32_t count);
/* Measurement aid for the latency of Early Inference Cancellation on the device clock: while
 * barrier tracing is on (pi_debug_set_plan phase 5), later forwards raise the cancel word of their
 * first run THEMSELVES -- a workgroup in the middle of the grid stores 1 into it when it enters
 * phase `phase` (0 QKV, 2 O, 3 gate/up, 4 down) of layer `layer`, then stamps the 100 MHz clock
 * into entry 5 * n_layers + 7 of the trace -- so the store comes from another compute unit than the
 * one that probes the word, at a known moment of a known layer.  The run must then stop at the
 * boundary that ends this layer: layers_done == layer + 1.  layer < 0 switches it off. */
int32_t pi_debug_raise_cancel(pi_model* m, int32_t layer, int32_t phase);
/* What a launch of the forward's shape (one workgroup of 8 waves per compute unit, rings of eight
 * 128-bit non-temporal loads per lane) reads per second when it does nothing else: allocates
 * `bytes` (>= 64 MiB) of device memory, streams it reps + 1 times and returns the best rate in
 * GB/s.  Blocking; frees what it allocated. */
int32_t pi_debug_stream_probe(int64_t bytes, int32_t reps, double* gbps);
/* Debug hook: per-workgroup timestamps of the five phases of one layer.  `layer` selects the layer
 * later runs record (-1: none).  With dst_host non-null, first copies the last recording to the
 * host: grid x 5 x 8 values of the 100 MHz clock, per workgroup and phase (0 QKV, 1 attention, 2 O,
 * 3 gate/up, 4 down): [0] phase entered, [2] the phase's work done (stores settled), [3] before
 * the barrier, [4] workgroup arrived at the barrier, [5] barrier passed (phases 2 and 4 end in a
 * barrier; the others hand over through the data).  Blocking. */
int32_t pi_debug_wgtrace(pi_model* m, int32_t layer, uint64_t* dst_host);

#ifdef __cplusplus
}
#endif
#endif /* PIPEINFER_H */
