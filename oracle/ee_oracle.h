/*
 * ee_oracle.h -- CPU oracle for the batched early-exit decode step.
 *
 * TEST INFRASTRUCTURE ONLY.  This is the plain, slow, obviously-correct
 * statement of what the early-exit decode step computes.  It exists so that
 * the GPU library can be checked against something that was written from the
 * paper and from the textbook definitions of the decoder primitives, and it
 * shares no code with that library.  Nothing on a product path may call it.
 *
 * What the paper fixes (HELIOS, arXiv 2504.10724):
 *   - a token leaves the layer stack at an exit layer when its probability
 *     meets a confidence threshold (Sec. 1, Sec. 2.1);
 *   - threshold 1 keeps every token in the stack, threshold 0 releases every
 *     token at the first exit (Sec. 3.1, Insight 2);
 *   - keys and values are still produced for the layers a token skipped,
 *     because later tokens that go deeper attend to every earlier token
 *     (Sec. 2.2);
 *   - with greedy partial loading only layers 1..R are resident and every
 *     token stops at layer R at the latest, confident or not (Sec. 3.3.3,
 *     Sec. 5.4); a token that stops there below the threshold is a
 *     "confidence breach" (Sec. 3.3.3, CBC).
 * Everything else (RMSNorm, rotary embedding, grouped-query attention,
 * SwiGLU) is the standard Llama-family decoder layer.
 *
 * Arithmetic: values are held in fp32; every dot product and every sum is
 * accumulated in fp64 and rounded once to fp32.  With dtype == ORC_BF16 the
 * operands of every matrix product (normalised activations, attention output,
 * SwiGLU product) and the cached K and V are rounded to bfloat16
 * (round-to-nearest-even) first; with dtype == ORC_F32 nothing is rounded.
 *
 * All pointers are host pointers owned by the caller.  Matrices are row-major
 * [out_features][in_features]; bf16 matrices are arrays of uint16_t holding
 * the upper 16 bits of the fp32 pattern.
 *
 * Pinned by tests/test_oracle_*.py; no function here is "parity unpinned".
 */
#ifndef EE_ORACLE_H
#define EE_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { ORC_F32 = 0, ORC_BF16 = 1 };
enum { ORC_OK = 0, ORC_ERR_ARG = -1, ORC_ERR_NOT_RESIDENT = -2 };

typedef struct {
    int32_t n_layers;   /* L: depth of the full model                          */
    int32_t d_model;    /* d                                                   */
    int32_t n_q_heads;  /* H_q                                                 */
    int32_t n_kv_heads; /* H_kv (H_q % H_kv == 0)                              */
    int32_t head_dim;   /* hd (even)                                           */
    int32_t d_ffn;      /* F                                                   */
    int32_t vocab;      /* V                                                   */
    int32_t dtype;      /* ORC_F32 or ORC_BF16                                 */
    float   rms_eps;
    int32_t n_exits;    /* number of exit heads of the full model              */
    int32_t exit_layers[16]; /* 1-based, ascending                             */
} orc_config;

typedef struct orc_model orc_model;

/* Key/value cache of the rows the oracle works on: dense, fp32 values,
 * K and V each [n_layers_resident][B][H_kv][cap][hd]. */
typedef struct {
    float*  K;
    float*  V;
    int32_t B;
    int32_t cap;
} orc_kv;

int orc_model_create(const orc_config* cfg, orc_model** out);
void orc_model_destroy(orc_model* m);
/* layer is 1-based.  W_qkv rows: H_q*hd query rows, then H_kv*hd key rows,
 * then H_kv*hd value rows.  Setting a layer makes it resident. */
int orc_model_set_layer(orc_model* m, int layer, const float* g_attn,
                        const void* W_qkv, const void* W_o, const float* g_ffn,
                        const void* W_gate, const void* W_up, const void* W_down);
int orc_model_set_exit(orc_model* m, int exit_idx, const float* g_exit, const void* W_exit);
int orc_model_set_embed(orc_model* m, const void* emb);
/* rotary base theta (10000 for the Llama family) and the largest position + 1 */
int orc_model_set_rope(orc_model* m, double theta, int max_pos);
/* deepest resident layer R if layers 1..R are exactly the resident ones, else -1 */
int orc_model_resident_depth(const orc_model* m);

/* ---- primitives (one row / one head), exposed so that tests can pin them ---- */
void  orc_round_bf16(float* x, size_t n);
void  orc_rmsnorm(const float* h, const float* g, int d, float eps, int round_bf16, float* out);
/* out[j] = sum_k x[k] * W[j][k], j < N */
void  orc_matvec(const float* x, const void* W, int dtype, int N, int K, float* out);
void  orc_rope(float* v, int hd, int pos, double theta);
/* one query head over n_pos cached positions: K, V are [n_pos][hd] */
void  orc_attention_head(const float* q, const float* K, const float* V, int n_pos, int hd, float* out);
float orc_silu(float t);
/* max-probability confidence and lowest-index argmax of z[0..V) */
void  orc_softmax_conf(const float* z, int V, float* conf, int32_t* tok);
/* order-preserving split of active[0..n) by exit_mask[0..n): survivors keep
 * their order in out_active, leavers keep theirs in out_exited */
void  orc_compact(const uint8_t* exit_mask, const int32_t* active, int n,
                  int32_t* out_active, int32_t* out_n, int32_t* out_exited, int32_t* out_m);

/* ---- the calls of the path ---- */
int orc_embed(const orc_model* m, int32_t tok, float* h_row);
/* one decoder layer on the rows with active[b] != 0; h is [B][d], in place;
 * appends K,V of the layer at position pos[b] */
int orc_layer_forward(const orc_model* m, int layer, orc_kv* kv, const uint8_t* active,
                      const int32_t* pos, float* h);
/* exit head of one row: logits (nullable, [V], already multiplied by scale) */
int orc_exit_head(const orc_model* m, int exit_idx, const float* h_row, float scale,
                  float* logits, float* conf, int32_t* tok);
/* K,V of layers (from_excl, to_incl] for row b from its exit hidden state */
int orc_fill_skipped_kv(const orc_model* m, int from_excl, int to_incl, orc_kv* kv,
                        int b, int32_t pos_b, const float* h_row);

/* One early-exit decode step over all B rows.
 *   thresholds[n_thresholds]: one per resident exit, ascending layer order.
 *   pos is advanced by one for every row.  counts[e] += rows that left at
 *   resident exit e.  layers_run (nullable): number of (row, layer) pairs
 *   executed.  h_out (nullable, [B][d]): each row's hidden state at its exit.
 *   conf_trace (nullable, [B][n_exits]): the confidence each row had at every
 *   exit it reached; entries of exits it did not reach are left untouched.
 */
int orc_decode_step(const orc_model* m, orc_kv* kv, const int32_t* tok_in, int32_t* pos,
                    const float* scale, const float* thresholds, int n_thresholds,
                    int32_t* out_tok, int32_t* out_layer, float* out_conf, uint8_t* out_breach,
                    int32_t* counts, int64_t* layers_run, float* h_out, float* conf_trace);

/* Full-depth decode with no exit logic at all: every row runs layers 1..R and
 * takes the token of the exit head at R.  Written separately from
 * orc_decode_step; used to pin the "threshold above 1" special case. */
int orc_vanilla_step(const orc_model* m, orc_kv* kv, const int32_t* tok_in, int32_t* pos,
                     const float* scale, int32_t* out_tok, float* out_conf, float* h_out);

/* Context pass ("prefill", the work that bounds the time to first token: Sec. 4.4,
 * Appendix E.1) of row b on the resident layers 1..R: the n tokens tok[0..n)
 * take positions pos0 .. pos0+n-1 (positions below pos0 must already be
 * cached).  Layer by layer over the whole context; within a layer position
 * pos0+t attends to positions 0 .. pos0+t only (causal), and its K, V are
 * appended.  No exit head runs: every context token passes all R layers, so
 * that a later token at any depth finds complete keys and values (Sec. 2.2).
 * h_out (nullable, [n][d]): hidden states after layer R. */
int orc_prefill(const orc_model* m, orc_kv* kv, int b, const int32_t* tok, int n, int32_t pos0,
                float* h_out);

/* Self-speculative decoding with one exit head as the drafter (Sec. 6: an early-exit model with an
 * intermediate exit below its loaded depth can also be served by exit-layer speculative decoding;
 * the scheme is the published draft-then-verify one, with the model's own first layers as the draft
 * model).  Acceptance rule alone: drafts d[0..k) against the full-depth tokens v[0..k) for the same
 * positions; with a = number of leading positions where they agree, the round emits
 * n = min(a + 1, k) tokens, namely v[0..n) (the accepted drafts, then the first correction).  Returns n. */
int orc_accept_drafts(const int32_t* drafts, const int32_t* verified, int k, int32_t* emitted);

/* One round for row b, written out step by step:
 *   1. draft: for j = 0..k-1 the input token (tok_in for j = 0, else draft j-1) at position pos+j runs
 *      layers 1..L_e (L_e = layer of exit `draft_exit`), which appends their K, V; its state after
 *      layer L_e is kept; exit head `draft_exit` gives draft j (greedy, lowest index on ties);
 *   2. verify: the k kept states run layers L_e+1..R, layer by layer and within a layer in rising
 *      position order (causal), appending those layers' K, V; the exit head at R gives verified[j];
 *   3. accept: orc_accept_drafts.  *pos advances by the number of emitted tokens; the input of the
 *      next round is the last emitted token.
 * What the scheme reaches is a plain definition: the emitted tokens and every cache entry below the
 * new position are those of full-depth greedy decoding (orc_vanilla_step), bit for bit here, whatever
 * k and draft_exit are; entries at positions from the new position on are leftovers of rejected drafts
 * and are overwritten when those positions are decoded.
 * drafts, verified, emitted: [k].  R must carry an exit head; L_e < R.
 * draft_margin, verify_margin (nullable, [k]; a diagnostic for comparisons, not part of the method):
 * for each head evaluation (largest logit - second largest logit) / largest |logit|, i.e. how far the
 * greedy choice is from a tie relative to the size of the logits. */
int orc_selfspec_round(const orc_model* m, orc_kv* kv, int b, int32_t tok_in, int32_t* pos, int draft_exit,
                       int k, int32_t* drafts, int32_t* verified, int32_t* n_emitted, int32_t* emitted,
                       float* draft_margin, float* verify_margin);

#ifdef __cplusplus
}
#endif
#endif
