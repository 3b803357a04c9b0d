/*
 * ee.h -- libee: the batched early-exit decode step on AMD MI355X (gfx950).
 *
 * One decode step produces one token for every request (row) of a batch.  Each
 * decoder layer runs only on the rows whose token is still in the layer stack;
 * at each exit layer an exit head gives every remaining token a confidence;
 * tokens whose confidence meets the threshold leave, and the layers they skip
 * still receive their keys and values.  The operations follow HELIOS
 * (arXiv 2504.10724): confidence-threshold early exit (Sec. 1, Sec. 2.1),
 * keys/values for skipped layers (Sec. 2.2), greedy partial loading with a
 * forced exit at the last resident layer (Sec. 3.3.3, Sec. 5.4) and the
 * per-token "confidence not met" signal that feeds the Confidence Breach
 * Counter (Sec. 3.3.3, Algorithm 1).  The decoder layer itself is the
 * Llama-family layer (RMSNorm, rotary embedding, grouped-query attention,
 * SwiGLU).
 *
 * Around the step, in the order of this file: the context pass that builds the
 * cache a step reads (ee_prefill); exit-layer self-speculative decoding on the
 * same kernels (ee_draft_step, ee_verify_drafts); loading further layers while steps run and
 * giving the cached tokens keys and values in them (ee_model_set_layer_on,
 * ee_hstore_*, ee_backfill_kv); and the two device-side records the serving
 * loop reads instead of per-row outputs, the confidence-breach counter
 * (ee_cbc_*) and the Performance History Table row (ee_pht_*).
 *
 * Conventions
 *   - Plain C ABI.  Every call returns EE_OK (0) or a negative ee_status;
 *     ee_last_error() gives a thread-local message for the last failure.
 *   - "dev" pointers are device (HBM) pointers, "host" pointers are host
 *     pointers.  The caller allocates and owns every large device buffer
 *     (weights, key/value pool, batch state, workspace); the library borrows
 *     them.  The library itself allocates only small per-handle tables (rotary
 *     table, row tables) when a handle is created or bound, never in a
 *     hot-path call.
 *   - Hot-path calls only enqueue kernels on `stream` (a hipStream_t passed as
 *     void*, NULL = the default stream) and return; results are valid after
 *     the caller synchronises the stream.  The number of active rows lives on
 *     the device, so no call waits for the GPU.
 *   - Layers are numbered from 1.  Exits are numbered from 0 in the order of
 *     ee_model_config.exit_layers.
 *   - There is no CPU fallback: without a gfx950 device every compute call
 *     fails with EE_ERR_HIP.
 *
 * Precision contract (dtype EE_BF16): weights, the embedding, cached K and V
 * and the left operand of every matrix product (normalised activations, the
 * attention output, the SwiGLU product) are bfloat16, rounded to nearest even;
 * products accumulate in fp32; the residual stream, queries, rotary
 * embedding, attention scores and softmax, SiLU, norm statistics and the
 * exit-head logits, scale and softmax are fp32.  dtype EE_F32 rounds nowhere.
 */
#ifndef EE_H
#define EE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define EE_MAX_EXITS 16

typedef enum {
    EE_OK = 0,
    EE_ERR_INVALID_ARG = -1,        /* null pointer, NaN threshold, wrong count ...          */
    EE_ERR_SHAPE = -2,              /* dimensions the kernels do not support                 */
    EE_ERR_CAPACITY = -3,           /* batch or buffer larger than what was bound            */
    EE_ERR_LAYER_NOT_RESIDENT = -4, /* layer was never set (not loaded)                      */
    EE_ERR_EXIT_NOT_RESIDENT = -5,  /* exit head not set, or deepest resident layer no exit  */
    EE_ERR_DTYPE = -6,
    EE_ERR_HIP = -7                 /* a HIP runtime call failed                             */
} ee_status;

typedef enum { EE_F32 = 0, EE_BF16 = 1 } ee_dtype;

typedef struct {
    int32_t n_layers;    /* L, depth of the full model                                      */
    int32_t d_model;     /* d                                                               */
    int32_t n_q_heads;   /* H_q                                                             */
    int32_t n_kv_heads;  /* H_kv, divides H_q; H_q / H_kv <= 16                             */
    int32_t head_dim;    /* hd; EE_BF16 requires 128, EE_F32 any even value <= 256          */
    int32_t d_ffn;       /* F                                                               */
    int32_t vocab;       /* V                                                               */
    int32_t dtype;       /* ee_dtype                                                        */
    float   rms_eps;
    float   rope_theta;  /* rotary base (10000 for the Llama family)                        */
    int32_t max_pos;     /* positions 0 .. max_pos-1 can be decoded                         */
    int32_t n_exits;     /* exit heads of the full model, <= EE_MAX_EXITS                   */
    int32_t exit_layers[EE_MAX_EXITS]; /* ascending, 1-based                                */
} ee_model_config;
/* EE_BF16 additionally requires d, F, H_q*hd multiples of 64 and (H_q+2H_kv)*hd, V
 * multiples of 32 (violations: EE_ERR_SHAPE). */

/* Device pointers to the weights of one layer.
 * EE_F32 : row-major [out_features][in_features] fp32, used in place.
 * EE_BF16: tile-packed bf16 produced by ee_pack_weight (see there).
 *   w_qkv : [(H_q + 2 H_kv) hd][d]; rows are H_q*hd query rows, then H_kv*hd key rows,
 *           then H_kv*hd value rows
 *   w_o   : [d][H_q hd]
 *   w_gate_up : EE_F32: [2F][d], the F gate rows followed by the F up rows;
 *               EE_BF16: the packed form of the [2F][d] matrix whose row 2j is gate row j and
 *               whose row 2j+1 is up row j (one lane of a matrix-core result then holds both)
 *   w_down: [d][F]
 *   g_attn, g_ffn: fp32 [d] RMSNorm gains. */
typedef struct {
    const float* g_attn;
    const void*  w_qkv;
    const void*  w_o;
    const float* g_ffn;
    const void*  w_gate_up;
    const void*  w_down;
} ee_layer_weights;

typedef struct ee_model ee_model;
typedef struct ee_kv    ee_kv;
typedef struct ee_batch ee_batch;

const char* ee_last_error(void);
/* Number of HIP devices visible, or a negative ee_status. */
int ee_device_count(void);

/* ------------------------------------------------------------------ weights */

/* Bytes of the packed form of an [n_out][n_in] bf16 matrix (= n_out*n_in*2). */
size_t ee_packed_bytes(int n_out, int n_in);

/* Repack rows of a row-major bf16 matrix src[n_out][n_in] (dev) into the tile order the MFMA
 * kernels stream.  The destination is the packed form of a [dst_rows][n_in] matrix D: it is cut
 * into tiles of 32 rows x 16 input columns; tile (r, c) sits at tile slot c * (dst_rows / 32) + r
 * (all tiles of one 16-column slice of K are contiguous) and is stored as 64 x 8 values where
 * entry (l, j) is D[32 r + l % 32][16 c + 8 (l / 32) + j].  Source row i becomes row
 * row_offset + i * row_stride of D.  (row_offset, row_stride, dst_rows) = (0, 1, n_out) packs a
 * matrix on its own; (0, 2, 2F) for the gate matrix and (1, 2, 2F) for the up matrix build
 * w_gate_up, in which gate row j and up row j are neighbours (rows 2j and 2j+1).
 * n_in % 16 == 0 and dst_rows % 32 == 0, else EE_ERR_SHAPE; a placement outside the destination
 * gives EE_ERR_INVALID_ARG.  Runs on `stream`; src may be freed after the stream is synchronised. */
int ee_pack_weight(const void* dev_src, int n_out, int n_in, void* dev_dst,
                   int row_offset, int row_stride, int dst_rows, void* stream);

/* ------------------------------------------------------------------ handles */

/* Creates a model description with no layer resident.  Builds the rotary
 * cos/sin table for positions < max_pos on the current device.  Set-up call:
 * it allocates the table and two per-layer pointer tables and waits for the
 * default stream (the table kernel) before it returns. */
int ee_model_create(const ee_model_config* cfg, ee_model** out);
int ee_model_destroy(ee_model* m);
/* Makes layer `layer` resident (Sec. 3.3.3: only the layers up to the chosen
 * exit are loaded).  The pointed-to buffers must outlive the model.  Set-up
 * call: the two device-side table entries are written with synchronous copies
 * (ee_model_set_layer_on is the variant that does not wait). */
int ee_model_set_layer(ee_model* m, int layer, const ee_layer_weights* dev_w);
/* Exit head exit_idx: fp32 gain [d] and W_exit [V][d] (packed if EE_BF16). */
int ee_model_set_exit(ee_model* m, int exit_idx, const float* dev_gain, const void* dev_w_exit);
/* Embedding [V][d], row-major in the model dtype (never packed). */
int ee_model_set_embed(ee_model* m, const void* dev_emb);
/* Deepest resident layer R if exactly layers 1..R are resident, else EE_ERR_INVALID_ARG. */
int ee_model_resident_depth(const ee_model* m);

/* Key/value pool.  Row b owns capacity[b] positions (EE_BF16: a multiple of 32)
 * and the rows are laid out back to back: with T_b = capacity[0]+..+capacity[b-1]
 * and T the sum over all rows, the block of (layer l, row b, kv-head g) starts at
 * element  ((l-1)*T + T_b) * 2*H_kv*hd + g * 2*capacity[b]*hd  and holds
 *   EE_F32 : K: capacity[b] x hd, position-major K[p][i]; V: the same, right after K
 *   EE_BF16: groups of 32 positions, each group 64*hd elements = [K of the group][V of the group],
 *            so that one (row, head) is a single contiguous stream.  With p = 32 q + r, relative
 *            to the block's start:
 *              K[p][i] at q*64*hd + ((((r/16)*4 + i/32) * 4 + (i%32)/8) * 16 + r%16) * 8 + i%8
 *              V[p][i] at q*64*hd + 32*hd + (((i/16)*4 + (r%16)/4) * 16 + i%16) * 8 + (r/16)*4 + r%4
 *   (both bf16 orders are the operand orders of the attention MFMAs; use
 *   ee_kv_write_context / ee_kv_read_context to convert from and to plain position-major data)
 * ee_kv_pool_bytes gives the size for R resident layers.  host_capacity is a
 * host array [B]; the library keeps a device copy. */
size_t ee_kv_pool_bytes(const ee_model* m, int n_resident_layers, const int32_t* host_capacity, int B);
int ee_kv_bind(const ee_model* m, void* dev_pool, size_t pool_bytes, int n_resident_layers,
               const int32_t* host_capacity, int B, ee_kv** out);
int ee_kv_destroy(ee_kv* kv);
/* Copy `n_pos` positions of plain position-major context into / out of the pool
 * layout for (layer, row): dev_k, dev_v are [H_kv][n_pos][hd] in the model dtype. */
int ee_kv_write_context(const ee_model* m, ee_kv* kv, int layer, int row, int pos0, int n_pos,
                        const void* dev_k, const void* dev_v, void* stream);
int ee_kv_read_context(const ee_model* m, const ee_kv* kv, int layer, int row, int pos0, int n_pos,
                       void* dev_k, void* dev_v, void* stream);

/* Batch state: residual stream, row lists, positions, outputs.  The caller
 * provides dev_state (ee_batch_state_bytes) and dev_workspace
 * (ee_workspace_bytes), both 256-byte aligned. */
size_t ee_batch_state_bytes(const ee_model* m, int B);
size_t ee_workspace_bytes(const ee_model* m, int B);
int ee_batch_bind(const ee_model* m, int B, void* dev_state, size_t state_bytes,
                  void* dev_workspace, size_t workspace_bytes, ee_batch** out);
int ee_batch_destroy(ee_batch* b);

/* Byte offsets of the fields of the batch state inside dev_state. */
typedef struct {
    size_t h;            /* fp32 [B][d]   residual stream, indexed by row id            */
    size_t tok_in;       /* int32 [B]     input token of the coming step                */
    size_t pos;          /* int32 [B]     position of that token (= cached positions)   */
    size_t row_scale;    /* fp32 [B]      multiplier of the exit-head logits            */
    size_t active_idx;   /* int32 [B]     row ids still in the stack, ascending         */
    size_t n_active;     /* int32         how many                                      */
    size_t exited_idx;   /* int32 [B]     row ids that left at the last compaction      */
    size_t n_exited;     /* int32                                                       */
    size_t head_conf;    /* fp32 [B]      last exit head: confidence of active_idx[i]   */
    size_t head_tok;     /* int32 [B]     last exit head: argmax token of active_idx[i] */
    size_t head_exit;    /* uint8 [B]     last exit head: 1 = leaves                    */
    size_t head_breach;  /* uint8 [B]     last exit head: leaves below the threshold    */
    size_t out_tok;      /* int32 [B]     emitted token per row id                      */
    size_t out_layer;    /* int32 [B]     layer the row left at (0 = not yet)           */
    size_t out_conf;     /* fp32 [B]      its confidence there                          */
    size_t out_breach;   /* uint8 [B]     1 = left at the last resident layer below th. */
    size_t exit_counts;  /* int32 [EE_MAX_EXITS] rows that left at each exit (cumulative) */
    size_t breach_count; /* int32         cumulative number of breaches                  */
    size_t status;       /* int32         0, or a bit set by a kernel that refused work: */
                         /*               1 = a row's position reached its capacity      */
                         /*               2 = an input token outside the vocabulary      */
} ee_batch_layout;
int ee_batch_get_layout(const ee_model* m, int B, ee_batch_layout* out);

/* Start from given tokens / positions / scales (device arrays [B]; dev_row_scale
 * may be NULL = 1.0): all B rows active, outputs and counters cleared. */
int ee_batch_reset(ee_batch* b, const int32_t* dev_tok_in, const int32_t* dev_pos,
                   const float* dev_row_scale, void* stream);
/* New per-row logit scales for the coming step. */
int ee_batch_set_row_scale(ee_batch* b, const float* dev_row_scale, void* stream);
/* All B rows active again, h = embedding of tok_in (what ee_decode_step does first). */
int ee_batch_begin_step(const ee_model* m, ee_batch* b, void* stream);

/* ------------------------------------------------------------------ hot path */

/* One decoder layer on the active rows (Sec. 5.1: time is layers traversed x
 * time per layer): h += Attn(RMSNorm(h)) W_o, then h += SwiGLU-FFN(RMSNorm(h));
 * appends the rows' K and V of this layer at their positions.
 * Errors: EE_ERR_LAYER_NOT_RESIDENT if the layer was never set. */
int ee_layer_forward(const ee_model* m, int layer, ee_kv* kv, ee_batch* b, void* stream);

/* Exit head `exit_idx` on the active rows (Sec. 2.1: a token leaves if its
 * probability meets the threshold): z = scale_b * (RMSNorm(h_b) W_exit),
 * confidence = max softmax probability, token = lowest-index argmax,
 * leaves = confidence >= threshold or force_exit (the layer is the last
 * resident one, Sec. 3.3.3), breach = force_exit and confidence < threshold.
 * Writes head_conf/head_tok/head_exit/head_breach for i < n_active.  Logits are
 * not stored unless dev_dbg_logits (fp32 [B][V], row i = active_idx[i]) is given. */
int ee_exit_head(const ee_model* m, int exit_idx, float threshold, int force_exit,
                 ee_batch* b, float* dev_dbg_logits, void* stream);

/* ee_exit_head for callers that cannot allocate device memory and bring no workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels, same
 * results (bit for bit) and same outputs in the batch state as ee_exit_head without the debug
 * pointer, but what that call keeps in the batch's workspace (normalised operand rows, per-tile
 * softmax statistics, for EE_F32 also the logits) goes to a device array of EE_STATIC_SCRATCH_BYTES
 * that the library holds on every GPU it runs on until the process ends.  The call allocates
 * nothing and frees nothing (its first call on a device looks the array's address up); the
 * batch's own workspace is not touched.  Nothing in the array has to start at zero: every value
 * read was written by this call.  All calls on one GPU share the array: calls that overlap in
 * time on one GPU (different streams or threads) race; calls on one stream are safe.  Kernel
 * timing (ee_timing_enable) creates events and must be off for a caller that may not allocate.
 * Errors as ee_exit_head; EE_ERR_CAPACITY if the batch and model need more than
 * EE_STATIC_SCRATCH_BYTES (about Mpad * (2 d + 12 V / 32) bytes for EE_BF16 with Mpad = the
 * batch's rows rounded up to 32: 7.2 MiB for 256 rows at d = 8192, V = 32000). */
#define EE_STATIC_SCRATCH_BYTES ((size_t)16 << 20)
int ee_exit_head_static(const ee_model* m, int exit_idx, float threshold, int force_exit, ee_batch* b,
                        void* stream);

/* The step that lets rows of one batch leave at different exits (Sec. 1: batching early-exit
 * requests needs the tokens of a batch kept in step; Sec. 5.4 removes the problem by making every
 * token of a batch stop at the same layer, here the batch is re-formed on the device instead).
 * Order-preserving compaction of the active rows by head_exit: survivors stay in
 * active_idx (ascending), leavers go to exited_idx; the leavers' token, layer,
 * confidence and breach flag are scattered to out_*[row id]; n_active, n_exited,
 * exit_counts[exit_idx] and breach_count are updated on the device. */
int ee_compact_active(ee_batch* b, int exit_idx, int exit_layer, void* stream);

/* K and V of layers (from_layer_excl, to_layer_incl] for the rows in exited_idx,
 * from their hidden state at the exit (Sec. 2.2: skipped layers still get their
 * KV): x = RMSNorm(h_b; g_attn of that layer), K = RoPE(x W_k, pos_b), V = x W_v. */
int ee_fill_skipped_kv(const ee_model* m, int from_layer_excl, int to_layer_incl,
                       ee_kv* kv, ee_batch* b, void* stream);

/* One whole early-exit decode step, i.e. one output token for every request of the batch
 * (Sec. 2.1: a token is emitted at the first exit whose confidence threshold it meets; Sec. 3.3.3 and
 * Sec. 5.4: at the last resident layer R in any case): embed tok_in; for l = 1..R run the layer on
 * the active rows and, where l carries an exit, the exit head, the compaction
 * and the fill of skipped layers; then pos += 1 and tok_in = out_tok for every
 * row.  When the step returns, every row has its K and V in all R layers, as if
 * ee_fill_skipped_kv(l, R) had run at each exit layer l; the bf16 step gets there
 * in segments (after the compaction at l: layers l+1 .. next exit layer, for all
 * rows that have left so far in this step), which reads each layer's W_k, W_v once.  host_thresholds holds one value per resident exit; values <= 0 always
 * exit, values > 1 never do (except at R).
 * Errors: EE_ERR_EXIT_NOT_RESIDENT if layer R carries no (set) exit head,
 * EE_ERR_INVALID_ARG if the resident layers are not exactly 1..R, if
 * n_thresholds differs from the number of resident exits or a threshold is NaN,
 * EE_ERR_CAPACITY if the cache was bound for fewer layers than R. */
int ee_decode_step(const ee_model* m, ee_kv* kv, ee_batch* b, const float* host_thresholds,
                   int n_thresholds, void* stream);

/* The same step in pieces, for callers that look at the batch between exits.  With one or a few
 * requests in the batch (the paper's default is one, Sec. 1) every row has often left well before
 * layer R, and the launches of the layers that no row reaches then cost more than a look at n_active:
 * segment e = the layers after exit e - 1 up to exit layer e (segment 0 starts with the embedding), exit
 * head e, the compaction, and the K/V of the layers up to the next exit for the rows that have left.
 * A step is ee_decode_segment for e = 0, 1, ... in order, then ee_decode_finish(last segment run); the
 * caller may stop after any segment once n_active is 0 (it reads that field itself, after synchronising
 * the stream), and must run all segments otherwise.  ee_decode_finish gives the rows that have left their
 * K and V in the layers of the segments that were not run, then pos += 1 and tok_in = out_tok as at the
 * end of ee_decode_step.  Outputs, cache and batch state are those of ee_decode_step, bit for bit.
 * Finishing while rows are still active leaves those rows without a token: the caller's error, not
 * detected here.  Errors: as ee_decode_step; EE_ERR_INVALID_ARG if there is no such segment. */
int ee_decode_segment(const ee_model* m, ee_kv* kv, ee_batch* b, const float* host_thresholds,
                      int n_thresholds, int segment, void* stream);
int ee_decode_finish(const ee_model* m, ee_kv* kv, ee_batch* b, int last_segment, void* stream);

/* Context pass ("prefill") on the resident layers 1..R: builds the keys and values that the
 * decode step reads; its duration is what bounds the time to first token (Sec. 4.4,
 * Appendix E.1), and with greedy partial loading it runs on R layers only (Sec. 3.3.3).
 * Entry i < n (device arrays of n int32 each) is token dev_tok[i] at position dev_pos[i] of
 * cache row dev_seq[i].  Every entry passes all R layers, no exit head runs (a later token
 * at any depth must find complete keys and values, Sec. 2.2); in each layer the entry's K
 * and V are appended at its position and it attends to positions 0 .. dev_pos[i] of its
 * cache row (causal).  Those positions must be in the cache already or be entries of this
 * same call; several cache rows may be mixed in one call, and a long context is passed in
 * several calls on one stream, in rising position order.  Two entries with the same (cache
 * row, position) race.  n <= B of the batch; the cache may have any number of rows.
 * The call uses the batch's state and workspace: tok_in, pos, active_idx, n_active and h of
 * rows < n are overwritten (h[i] = entry i's hidden state after layer R), so a batch that
 * decodes is given its rows again with ee_batch_reset afterwards.  Refusals are reported in
 * the batch's status word: 1 = a position outside its cache row's capacity or a cache row
 * that does not exist, 2 = a token outside the vocabulary.  Enqueue-only, like the rest.
 * Errors: EE_ERR_CAPACITY if n > B or the cache holds fewer than R layers,
 * EE_ERR_LAYER_NOT_RESIDENT / EE_ERR_INVALID_ARG as for ee_decode_step. */
int ee_prefill(const ee_model* m, ee_kv* kv, ee_batch* b, const int32_t* dev_tok,
               const int32_t* dev_pos, const int32_t* dev_seq, int n, void* stream);

/* ------------------------------------------------------------------ exit-layer self-speculative decoding
 *
 * An early-exit model with an exit below its loaded depth can also be served by speculative decoding
 * with that exit as the drafter (Sec. 6, comparison with speculative decoding): the first layers and
 * their exit head draft k tokens one by one, the remaining layers check all k positions in one pass,
 * and the longest agreeing prefix is kept.  The emitted tokens are those of full-depth greedy decoding
 * (exit head at the last resident layer R); the gain is that the deep layers run once per round over
 * k positions instead of once per token.  One round on a batch of B rows:
 *     k times:  ee_draft_step, then ee_hstore_put_step (keeps each row's state after the draft layers)
 *     once:     ee_verify_drafts
 *     once:     ee_hstore_put_prefill on the entries batch, B * k entries (optional: replaces the kept
 *               states by those after layer R, which is what ee_backfill_kv needs if further layers
 *               are loaded later; positions beyond the emitted ones are written again by later rounds)
 */

/* One draft token for every row: embeds tok_in, runs layers 1 .. exit_layers[draft_exit] on all rows
 * (their K, V are appended), takes the greedy token of that exit head (lowest index on ties), then
 * pos += 1 and tok_in = the draft.  Deeper layers are not touched and get no K, V here.  out_tok,
 * out_conf and out_layer hold the draft, its probability and the draft layer; h holds each row's state
 * after the draft layers; the batch's exit counters count the drafts like exits and mean nothing
 * during a round.  dev_draft_out (nullable): B int32, receives the drafts.
 * Errors: as ee_decode_step; EE_ERR_INVALID_ARG if the draft exit is not below the deepest resident
 * layer; EE_ERR_EXIT_NOT_RESIDENT if the draft head or the head of the deepest resident layer is not set. */
int ee_draft_step(const ee_model* m, ee_kv* kv, ee_batch* b, int draft_exit, int32_t* dev_draft_out, void* stream);

/* Verification of k drafts per row.  b: the batch that made k ee_draft_step calls since its last emitted
 * token (its pos is k ahead).  vb: a second batch of the same model with at least B * k rows, used as
 * the list of entries (its state and workspace are overwritten); entry r * k + j is cache row r at
 * position pos[r] - k + j with the state kept in dev_store (see ee_hstore_bytes) as its residual stream.
 * All entries pass layers exit_layers[draft_exit] + 1 .. R in one pass (causal within a row, K and V of
 * those layers appended), the exit head at R gives each entry's full-depth token v_j, and with a = the
 * number of leading positions where draft and full-depth token agree the row emits n = min(a + 1, k)
 * tokens v_0 .. v_{n-1}.  Outputs: dev_n_emit [B] = n; dev_emit [B][k] = the emitted tokens, -1 beyond n;
 * b's pos = position before the drafts + n, tok_in = out_tok = v_{n-1}.  Cache entries from the new
 * position on are leftovers of rejected drafts and are overwritten when those positions are decoded.
 * dev_drafts: [k][B] int32, draft j of row r at j * B + r (what ee_draft_step wrote).
 * Afterwards vb holds the entries like a batch after ee_prefill (h = state after layer R, position and
 * cache row of every entry), so ee_hstore_put_prefill(m, kv, vb, B * k, ...) may follow.
 * Refusals (a position outside its cache row) set status bit 1 of vb.  Enqueue-only.
 * Errors: as ee_draft_step; EE_ERR_CAPACITY if vb has fewer than B * k rows; EE_ERR_INVALID_ARG on null
 * arrays, k < 1 or vb == b. */
int ee_verify_drafts(const ee_model* m, ee_kv* kv, ee_batch* b, ee_batch* vb, int draft_exit, int k,
                     const float* dev_store, const int32_t* dev_drafts, int32_t* dev_n_emit, int32_t* dev_emit,
                     void* stream);

/* ------------------------------------------------------------------ loading more layers while serving
 *
 * With greedy partial loading only layers 1..R are resident; when too many tokens stop at R below
 * their threshold the serving loop may load further layers of the same model (Sec. 3.3.3, "Load More
 * Layers Or Another Candidate Model?").  Two things are needed besides the weights: the new layers'
 * table entries must change without stopping the steps in flight, and the tokens that are cached
 * already need keys and values in the new layers (Sec. 2.2).  Those come from each token's hidden
 * state where it left the stack (a layer it did not run leaves that state unchanged), the same
 * rule as ee_fill_skipped_kv, so the states are kept in a store beside the cache.
 *
 * Store: device memory owned by the caller, fp32 [T][d_model], T = sum of the cache rows'
 * capacities; the state of position p of cache row r is at row (positions of rows before r) + p. */

/* As ee_model_set_layer, but the device-side table entries are written by a kernel on `stream`:
 * nothing waits on the host.  The caller orders the arrival of the weights before this call's
 * stream position (an event of the copy stream, say); steps enqueued on `stream` afterwards see
 * the layer. */
int ee_model_set_layer_on(ee_model* m, int layer, const ee_layer_weights* dev_w, void* stream);

/* Bytes of the exit-state store for this cache; 0 on a null handle. */
size_t ee_hstore_bytes(const ee_model* m, const ee_kv* kv);
/* After ee_decode_step: keeps h of every row (its state where it left) at the position the step
 * served (pos - 1 after the step).  Enqueue only.  A position outside the capacity sets status bit 1. */
int ee_hstore_put_step(const ee_model* m, const ee_kv* kv, const ee_batch* b, float* dev_store, void* stream);
/* After ee_prefill of n entries on this batch: keeps h of entry i (its state after layer R) at
 * (cache row, position) of the entry. */
int ee_hstore_put_prefill(const ee_model* m, const ee_kv* kv, const ee_batch* b, int n, float* dev_store,
                          void* stream);
/* K and V of layers (from_layer_excl, to_layer_incl] for n cached tokens, entry i = position
 * dev_pos[i] of cache row dev_seq[i], from their states in the store:
 * x = RMSNorm(state; g_attn of the layer), K = RoPE(x W_k, position), V = x W_v, written at the
 * token's position.  n <= B of the batch; the batch's h, pos, exited_idx and n_exited are
 * overwritten (use a batch that is not in the middle of a step, or reset it afterwards).
 * The layers' table entries are read on the device: enqueue this on the stream ee_model_set_layer_on
 * was given (or order it after that stream).
 * Errors as ee_fill_skipped_kv; EE_ERR_CAPACITY if n > B.  Refusals (no such cache row, position
 * outside its capacity) set status bit 1 and write nothing for that entry. */
int ee_backfill_kv(const ee_model* m, int from_layer_excl, int to_layer_incl, ee_kv* kv, ee_batch* b,
                   const float* dev_store, const int32_t* dev_pos, const int32_t* dev_seq, int n, void* stream);

/* ------------------------------------------------------------------ confidence-breach counter
 *
 * The serving loop above the decode step re-assesses its choice of model (load more
 * layers or switch) only when more than cbc_max of the last `window` emitted tokens
 * stopped below their confidence threshold (Sec. 3.3.3 and Algorithm 1 of the paper;
 * defaults 100 and 50).  The counter lives on the device so that no step has to wait
 * for the host: tokens are taken in the order (decode step, row id); the window holds
 * the most recent `window` tokens since the last re-assessment; after every token the
 * breaches in the window are compared with cbc_max; "more than" is strict; a
 * re-assessment empties the window.
 *
 * State: device memory owned by the caller, ee_cbc_state_bytes(window) bytes, 8-byte
 * aligned: this header followed by uint8 ring[window].  The host reads n_triggers (and
 * trigger_at) after synchronising the stream. */
#define EE_CBC_LOG 64
#define EE_CBC_MAX_WINDOW 4096
typedef struct {
    int32_t window;                 /* tokens in the sliding window                         */
    int32_t cbc_max;                /* breaches tolerated inside the window                 */
    int32_t head;                   /* ring slot the next token goes to                     */
    int32_t filled;                 /* tokens in the window (<= window)                     */
    int32_t count;                  /* breaches among them                                  */
    int32_t n_triggers;             /* re-assessments fired since ee_cbc_init               */
    int64_t tokens_seen;            /* tokens fed since ee_cbc_init                         */
    int64_t trigger_at[EE_CBC_LOG]; /* 1-based ordinal of the token of each of the first
                                       EE_CBC_LOG re-assessments                            */
} ee_cbc_state;

/* Bytes of a counter state for the given window; 0 if window is outside 1..EE_CBC_MAX_WINDOW. */
size_t ee_cbc_state_bytes(int window);
/* Writes a fresh state (enqueue only).  EE_ERR_INVALID_ARG on a null pointer, a window outside
 * 1..EE_CBC_MAX_WINDOW or a negative cbc_max. */
int ee_cbc_init(void* dev_state, int window, int cbc_max, void* stream);
/* Feeds n tokens: dev_flags[j] != 0 means token j stopped below its threshold.  Enqueue only. */
int ee_cbc_push(void* dev_state, const uint8_t* dev_flags, int n, void* stream);
/* Feeds the tokens of the decode step that just ran on this batch: out_breach[0 .. B). */
int ee_cbc_push_step(void* dev_state, const ee_batch* b, void* stream);

/* ------------------------------------------------------------------ Performance History Table row
 *
 * The serving loop keeps, per model, the early-exit profile (how many tokens left at each
 * exit), the accuracy estimate and the throughput of the requests it served (Sec. 3.3.2,
 * "Performance History Table"); accuracy is the perplexity of the generated tokens, taken from
 * the token probabilities alone (Sec. 4.4, Appendix A).  This row accumulates the device-side
 * part after each decode step, so that the host reads one small struct per window instead of
 * the per-row outputs of every step: tokens, exits[e] (e indexes ee_model_config.exit_layers),
 * breaches, and nll = sum of -ln p over the tokens, p = out_conf = the probability the exit head
 * gave the emitted token; perplexity = exp(nll / tokens).  Throughput is tokens over the wall time
 * the caller measures.  The sum runs in fp64 in a fixed order (bitwise repeatable).
 * State: sizeof(ee_pht_row) bytes of device memory owned by the caller, 8-byte aligned. */
typedef struct {
    int64_t tokens;
    int64_t breaches;
    int64_t exits[EE_MAX_EXITS];
    double  nll;
} ee_pht_row;
/* Zeroes the row (enqueue only). */
int ee_pht_init(void* dev_row, void* stream);
/* Adds the B tokens of the decode step that just ran on this batch (out_layer, out_conf,
 * out_breach); a row whose out_layer is not an exit layer of the model (it has not left) is
 * skipped.  Enqueue only.  EE_ERR_INVALID_ARG on a null pointer or a batch of another model. */
int ee_pht_push_step(void* dev_row, const ee_model* m, const ee_batch* b, void* stream);

/* ------------------------------------------------------------------ measurement aid */

/* Kernel classes of the decode step, for ee_timing_read. */
typedef enum {
    EE_K_EMBED = 0,     /* step begin: embedding gather                               */
    EE_K_NORM = 1,      /* RMSNorm -> matrix-product operand                          */
    EE_K_GEMM_QKV = 2,
    EE_K_ROPE_APPEND = 3,
    EE_K_ATTENTION = 4,
    EE_K_GEMM_O = 5,
    EE_K_GEMM_GATE_UP = 6,  /* with the SwiGLU epilogue                               */
    EE_K_GEMM_DOWN = 7,
    EE_K_EXIT_GEMM = 8,     /* vocabulary product with the fused softmax statistics   */
    EE_K_EXIT_DECIDE = 9,
    EE_K_COMPACT = 10,
    EE_K_FILL_KV = 11,      /* all kernels of ee_fill_skipped_kv                      */
    EE_K_CBC = 12,          /* confidence-breach counter update                       */
    EE_K_PHT = 13,          /* Performance History Table row update                   */
    EE_K_COUNT = 14
} ee_kernel_class;

/* class_mask: bit k set = every launch of kernel class k is bracketed by a pair of
 * HIP events recorded on the launch stream (this creates events: not for code
 * under graph capture); 0 = off, (1 << EE_K_COUNT) - 1 = all classes.  An event
 * pair costs a few microseconds of stream time, so time few classes when the
 * whole step is being measured as well.  ee_timing_read waits for the recorded
 * events, returns the number of launches and their summed duration in
 * milliseconds, and keeps accumulating until ee_timing_reset. */
int ee_timing_enable(int class_mask);
int ee_timing_reset(void);
int ee_timing_read(int kernel_class, int* launches, float* total_ms);

#ifdef __cplusplus
}
#endif
#endif
