/*
 * hexgen.h -- C ABI of the per-GPU pipeline-stage forward for MI355X (gfx950).
 *
 * One handle = one GPU's share of one pipeline stage of an asymmetric tensor+pipeline
 * parallel decoder (paper Section 3): `n_layers` consecutive Llama-2-style layers at
 * tensor-parallel degree `tp_degree`, rank `tp_rank` (paper Section 2, "Parallelism in
 * generative inference": weights split column-wise then row-wise, two all-reduce points per
 * layer).  The stage is run as prefill and then token-by-token decode against a KV cache
 * (paper Section 2, prefill / decode equations) and returns its PRE-ALL-REDUCE partial hidden
 * states.  Cross-GPU communication is not part of this library.
 *
 * Conventions
 *   - every call returns a status and never throws or aborts; out-params are untouched on error;
 *   - "device pointer" = HIP device memory of the current device, "host pointer" = ordinary
 *     host memory; the library never takes ownership of a caller buffer;
 *   - the library owns its copy of the weights (repacked), the KV cache and its workspace;
 *   - kernels are enqueued on `stream` (a hipStream_t passed as void*, NULL = default stream)
 *     and the call returns without synchronising, except where stated;
 *   - calls on one stage / cache are not thread-safe;
 *   - weights use the paper's x . W convention (Section 2): W is [in, out], row-major.
 *   - `dtype` fixes the storage type of weights, stage inputs / outputs and the KV cache.
 *     The residual stream, every accumulator, the softmax and the norm statistics are fp32.
 */
#ifndef HEXGEN_H
#define HEXGEN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hexgen_stage    hexgen_stage_t;     /* opaque, library-owned */
typedef struct hexgen_kv_cache hexgen_kv_cache_t;  /* opaque, library-owned */

/* Storage / operand type of weights, activations handed to the matrix cores and the KV cache; accumulation, norms,
 * softmax and the residual stream are fp32 for every value.  HEXGEN_F16 is the 2-byte precision the cost model's
 * B_type example names (Section 4.1 / Appendix B); HEXGEN_BF16 is the same path with the other 16-bit format. */
typedef enum { HEXGEN_F32 = 0, HEXGEN_BF16 = 1, HEXGEN_F16 = 2 } hexgen_dtype_t;

typedef enum {
    HEXGEN_OK = 0,
    HEXGEN_ERR_INVALID_ARG = 1, /* null pointer, negative size, unknown enum, index out of range */
    HEXGEN_ERR_SHAPE       = 2, /* sharding does not divide, unsupported head_dim / alignment       */
    HEXGEN_ERR_STATE       = 3, /* weights not loaded, decode before prefill, step mismatch        */
    HEXGEN_ERR_CAPACITY    = 4, /* KV overflow (len + new > max_seq), batch > max_batch            */
    HEXGEN_ERR_OOM         = 5, /* device or host allocation failed                                */
    HEXGEN_ERR_DEVICE      = 6  /* a HIP call failed                                               */
} hexgen_status_t;

const char *hexgen_status_string(hexgen_status_t s);

/* ---- stage ---------------------------------------------------------------------------------
 * Dimensions are GLOBAL (unsharded): a stage is (layers, tensor-parallel degree) as in paper
 * Section 3 / Section 4.1 (each stage has its own layer count l_ij and degree |d_ij|).  The
 * library derives head_dim = hidden / n_heads and rank `tp_rank`'s shard: query heads
 * [r*hq/t, (r+1)*hq/t), KV heads [r*hkv/t, (r+1)*hkv/t), FFN columns [r*F/t, (r+1)*F/t).
 * HEXGEN_ERR_SHAPE unless hidden % n_heads == 0, n_heads % n_kv_heads == 0, n_heads, n_kv_heads
 * and ffn divisible by tp_degree, 0 <= tp_rank < tp_degree, head_dim in {64, 128}, and (bf16, fp16)
 * hidden a multiple of 128, local q width and local ffn multiples of 32.  Defaults: rms_eps 1e-5, rope_theta 1e4.
 */
hexgen_status_t hexgen_stage_create(int hidden, int n_heads, int n_kv_heads, int ffn, int n_layers,
                                    int tp_degree, int tp_rank, hexgen_dtype_t dtype,
                                    hexgen_stage_t **out);
/* Call set_params before hexgen_kv_cache_create: a cache carries rotation tables built for the rope_theta of that
 * moment, and prefill / decode / run_sublayer return HEXGEN_ERR_STATE for a cache created under another rope_theta. */
hexgen_status_t hexgen_stage_set_params(hexgen_stage_t *st, float rms_eps, float rope_theta);
void            hexgen_stage_destroy(hexgen_stage_t *st);

/* Full (unsharded) matrices of one layer, row-major [in, out]:
 *   g_attn [H], wq [H, hq*d], wk [H, hkv*d], wv [H, hkv*d], wo [hq*d, H], g_ffn [H],
 *   w1 [H, F] (gate), w3 [H, F] (up), w2 [F, H] (down); element type = the stage's dtype
 *   (fp32, or bf16 / fp16 as raw 16-bit values).  Pointers may be host or device memory (detected).
 * The library copies rank r's shard (columns of wq/wk/wv/w1/w3, rows of wo/w2) and repacks it;
 * the call synchronises the device before returning, the sources may be freed afterwards.
 */
hexgen_status_t hexgen_stage_load_layer(hexgen_stage_t *st, int layer, const void *g_attn,
                                        const void *wq, const void *wk, const void *wv,
                                        const void *wo, const void *g_ffn, const void *w1,
                                        const void *w3, const void *w2);

/* ---- KV cache (paper Section 2: K, V of every processed position are kept per layer and the
 * new token's K, V are concatenated at each decode step) ---------------------------------------
 * Room for `max_batch` sequences of up to `max_seq` positions, for every layer of the stage.
 */
hexgen_status_t hexgen_kv_cache_create(hexgen_stage_t *st, int max_batch, int max_seq,
                                       hexgen_kv_cache_t **out);
void            hexgen_kv_cache_destroy(hexgen_kv_cache_t *kv);
/* Forget all sequences (lengths to 0, "not prefilled"). */
hexgen_status_t hexgen_kv_cache_reset(hexgen_kv_cache_t *kv);

/* ---- prefill (paper Section 2, prefill equations) ------------------------------------------
 * Packed (varlen) rows: sequence i occupies rows [cu_i, cu_i + seq_lens[i]) with cu the running
 * sum, at positions 0 .. seq_lens[i]-1.  Starts a new batch: the cache is reset first.
 *   hidden_in   device [total_rows, hidden], dtype           (activations from the previous stage)
 *   seq_lens    HOST int32 [batch], every entry >= 1
 *   out_partial device [total_rows, hidden], dtype: last layer's FFN partial P_ffn^(r), no residual
 *   out_resid   device [total_rows, hidden], dtype, may be NULL: the residual stream that partial
 *               would be added to; out_resid + sum over ranks of out_partial = the stage output
 * Interior reduce points (2 per layer, all-reduce in the paper) run in "solo" mode: the rank adds
 * its own partial to the residual stream, which is what one GPU can compute on its own; the kernel
 * shapes and bytes are those of the real sharded stage.
 */
hexgen_status_t hexgen_stage_prefill(hexgen_stage_t *st, hexgen_kv_cache_t *kv, const void *hidden_in,
                                     const int32_t *seq_lens, int batch, void *out_partial,
                                     void *out_resid, void *stream);

/* ---- decode (paper Section 2, decode equations) --------------------------------------------
 * One new row per sequence of the prefilled batch, at position len_i; K, V of the row are
 * appended.  `step` (0-based) must equal the number of decode calls since the prefill (or the
 * last hexgen_kv_cache_set_lengths), else HEXGEN_ERR_STATE.  Buffers as for prefill with
 * total_rows = batch.
 */
hexgen_status_t hexgen_stage_decode(hexgen_stage_t *st, hexgen_kv_cache_t *kv, int step,
                                    const void *hidden_in, void *out_partial, void *out_resid,
                                    void *stream);

/* ---- decode for callers that cannot allocate ------------------------------------------------------------------
 * For callers that may not call hipMalloc while they run: code under HIP graph capture, tight serving loops, harnesses
 * that forbid allocation.  Same step, same kernels and same results as hexgen_stage_decode, but the call allocates
 * nothing and frees nothing (no device memory, no host memory, no events): the workspace of the step -- residual
 * stream, projection operands, split partial sums of the batched projections, split-attention partials and arrival
 * counters, sums of squares, row positions -- is laid out in one file-scope device array of
 * HEXGEN_STATIC_SCRATCH_BYTES that every GPU the library runs on holds until the process ends.
 *   - bf16 and fp16 stages only (HEXGEN_ERR_SHAPE otherwise); at most 32 sequences in the batch, and the workspace of the
 *     call (hexgen_stage_decode_static_bytes(st, batch)) must fit the array: HEXGEN_ERR_CAPACITY otherwise, nothing
 *     is launched.  Every 70B-shaped configuration up to the full-width stage at batch 32 (39 MB) fits.
 *   - the cache must have been prefilled (or set_lengths called) as for hexgen_stage_decode; `step` as there; the
 *     cache, the lengths and the step count advance exactly as there, and the two calls may be mixed step by step.
 *   - all calls on one GPU share that GPU's array, which keeps the last call's contents; the call clears (with a
 *     kernel on `stream`) what has to start at zero.  Calls that overlap in time on one GPU -- two streams, two
 *     stages, two threads -- race on it: serialise them.
 *   - the timing slots of hexgen_stage_profile_enable are not recorded for this call; taps are.
 * hexgen_stage_decode_static_bytes: bytes of the array a call with `batch` sequences uses; -1 for invalid arguments
 * or an fp32 stage.
 */
#define HEXGEN_STATIC_SCRATCH_BYTES (64u << 20)
hexgen_status_t hexgen_stage_decode_static(hexgen_stage_t *st, hexgen_kv_cache_t *kv, int step,
                                           const void *hidden_in, void *out_partial, void *out_resid,
                                           void *stream);
int64_t hexgen_stage_decode_static_bytes(const hexgen_stage_t *st, int batch);

/* ---- validation surface ("group" mode: all t ranks of a stage run one after another on the same
 * GPU and their partials are summed, standing in for the all-reduce of paper Section 2) ----------
 * hexgen_stage_run_sublayer: one sub-layer of one layer for this rank.
 *   which 0: attention sub-layer  (RMSNorm, QKV, RoPE, cache append, attention, W_O partial)
 *   which 1: FFN sub-layer        (RMSNorm, W1/W3, SwiGLU, W2 partial)
 *   h_in        device fp32 [n_rows, hidden]: the residual stream entering the sub-layer
 *   seq_lens    HOST int32 [batch] rows per sequence (packed as in prefill), or NULL = one row
 *               per sequence for the first `batch` sequences (decode).  Rows of sequence i sit at
 *               positions len_i .. len_i + n_i - 1 where len_i is the committed length.
 *   partial_out device fp32 [n_rows, hidden]: this rank's partial (no residual)
 * The attention sub-layer writes K, V of the new rows into `layer`'s cache but does not change
 * the committed lengths; call hexgen_kv_cache_commit once all layers have processed the rows.
 */
hexgen_status_t hexgen_stage_run_sublayer(hexgen_stage_t *st, hexgen_kv_cache_t *kv, int layer,
                                          int which, const void *h_in, const int32_t *seq_lens,
                                          int batch, void *partial_out, void *stream);
hexgen_status_t hexgen_kv_cache_commit(hexgen_kv_cache_t *kv, const int32_t *seq_lens, int batch);
/* dst[i] += src[i] for n fp32 device elements (fixed-order rank sum of the validation driver). */
hexgen_status_t hexgen_accumulate_f32(void *dst, const void *src, int64_t n, void *stream);

/* Read back / install cache rows as HOST fp32 [n, hkv_local, head_dim] (K after rotation).
 * Both synchronise.  fill: sets positions 0..n-1 of `seq` in `layer`; when every layer of every
 * sequence of a batch has been filled, call hexgen_kv_cache_set_lengths to declare the context
 * (this also marks the cache "prefilled" and restarts the decode step count at 0).
 */
hexgen_status_t hexgen_kv_cache_read(hexgen_kv_cache_t *kv, int layer, int seq, int pos0, int n,
                                     float *k_out, float *v_out);
hexgen_status_t hexgen_kv_cache_fill(hexgen_kv_cache_t *kv, int layer, int seq, int n,
                                     const float *k, const float *v);
hexgen_status_t hexgen_kv_cache_set_lengths(hexgen_kv_cache_t *kv, const int32_t *lens, int batch);
hexgen_status_t hexgen_kv_cache_get_lengths(hexgen_kv_cache_t *kv, int32_t *lens_out, int batch);

/* Debug tap: at the entry of `layer` during prefill / decode, the fp32 residual stream
 * [rows, hidden] is copied to `h_dump` (device).  NULL removes the tap.
 */
hexgen_status_t hexgen_stage_set_tap(hexgen_stage_t *st, int layer, void *h_dump);

/* ---- the model's ends, adjacent to the first and the last stage -------------------------------------------
 * Paper Section 2: a request enters as prompt tokens and leaves as generated tokens, one per decode step.  These
 * calls turn a chain of stages into a token-in / token-out pipeline: the first stage's input rows come from the
 * embedding table, the last stage's output goes through the final RMSNorm and the LM head, and the next token is
 * the arg-max of the logits (greedy decoding).
 *
 * hexgen_embed_rows: rows_out[i] = table[tokens[i]].  table: device [vocab, hidden] row-major in `dtype`; tokens:
 * device int32 [n] (ids outside [0, vocab) are clamped); rows_out: device [n, hidden] in `dtype`, caller-owned.
 *
 * hexgen_head: vocabulary-parallel over tp_degree ranks (vocab divisible by it, else HEXGEN_ERR_SHAPE); rank tp_rank
 * holds columns [r V/t, (r+1) V/t) of the untied LM head.  hidden: multiple of 128 (bf16, fp16) or 4 (f32).
 * hexgen_head_load: g_final [hidden] and the FULL matrix w_lm [hidden, vocab], row-major, host or device, in the head's
 * dtype; the library copies and repacks its shard, the caller keeps its buffers.
 * hexgen_head_greedy: x = hidden_a (+ hidden_b when not NULL: e.g. a stage's out_resid and out_partial), device
 * [n_rows, hidden] in the head's dtype; per row: RMSNorm with g_final, this rank's logits, and the rank's best
 * candidate: token_out[i] = GLOBAL id (lowest id wins ties), logit_out[i] = its logit in fp32 (may be NULL).  Both are
 * device arrays of n_rows entries, caller-owned.  With tp_degree > 1 the caller picks, per row, the candidate with the
 * largest logit over the ranks (first maximum in rank order).  Enqueues on `stream`, does not synchronise.
 * HEXGEN_ERR_STATE before hexgen_head_load.
 */
typedef struct hexgen_head hexgen_head_t;
hexgen_status_t hexgen_embed_rows(const void *table, hexgen_dtype_t dtype, int hidden, int vocab, const int32_t *tokens,
                                  int n, void *rows_out, void *stream);
hexgen_status_t hexgen_head_create(int hidden, int vocab, int tp_degree, int tp_rank, hexgen_dtype_t dtype, float rms_eps,
                                   hexgen_head_t **out);
hexgen_status_t hexgen_head_load(hexgen_head_t *hd, const void *g_final, const void *w_lm);
hexgen_status_t hexgen_head_greedy(hexgen_head_t *hd, const void *hidden_a, const void *hidden_b, int n_rows,
                                   int32_t *token_out, float *logit_out, void *stream);
void            hexgen_head_destroy(hexgen_head_t *hd);

/* ---- the paper's cost model (Table 1; Appendix "Modeling the Generative Inference Cost", Eqs. 3-6) -----------
 * Host functions, plain arithmetic in double precision, no device work, thread-safe.  Task t = (batch b, prompt
 * length s_in, generated tokens s_out); bytes_per_elem = B_type; a stage = `layers` layers on n_dev devices with
 * memory bandwidths m_d[n_dev] (bytes/s) and peak rates c_d[n_dev] (flop/s), HOST arrays.  params_factor = parameters
 * of one layer in units of hidden^2: 12 for the paper's layer (its Eq. 3), 12.75 for Llama-2-70B's GQA + SwiGLU layer.
 * Every function returns seconds (hexgen_cost_mem: bytes), or NaN for an invalid argument (non-positive size or rate,
 * NULL array).
 *   hexgen_cost_comp         Eq. 3: max_d(P B s_out / (|d| m_d)) l + max_d(2 P b (s_in + s_out) / (|d| c_d)) l, P = params
 *   hexgen_cost_comp_prefill   its prefill share, 2 P b s_in / (|d| c_d) per layer
 *   hexgen_cost_comp_decode    its decode share, (P B / (|d| m_d) + 2 P b / (|d| c_d)) per layer and generated token
 *   hexgen_cost_comm_tp      Eq. 4: alpha, beta = n_dev x n_dev row-major link latencies (s) and bandwidths (bytes/s);
 *                            four supersteps per layer, the slowest device's sum per superstep; 0 for one device
 *   hexgen_cost_comm_pp      Eq. 5: alpha, beta = n_from x n_to links between the two stages; the fastest link carries
 *                            the prompt's activation once and one row per generated token
 *   hexgen_cost_mem          Eq. 6: parameters and K / V of the stage's layers split over the devices, plus four
 *                            activation buffers of b (s_in + s_out) hidden elements
 */
double hexgen_cost_comp(int hidden, double params_factor, int bytes_per_elem, int batch, int s_in, int s_out, int layers,
                        int n_dev, const double *m_d, const double *c_d);
double hexgen_cost_comp_prefill(int hidden, double params_factor, int bytes_per_elem, int batch, int s_in, int s_out,
                                int layers, int n_dev, const double *m_d, const double *c_d);
double hexgen_cost_comp_decode(int hidden, double params_factor, int bytes_per_elem, int batch, int s_in, int s_out,
                               int layers, int n_dev, const double *m_d, const double *c_d);
double hexgen_cost_comm_tp(int hidden, int bytes_per_elem, int batch, int s_in, int s_out, int layers, int n_dev,
                           const double *alpha, const double *beta);
double hexgen_cost_comm_pp(int hidden, int bytes_per_elem, int batch, int s_in, int s_out, int n_from, int n_to,
                           const double *alpha, const double *beta);
double hexgen_cost_mem(int hidden, double params_factor, int bytes_per_elem, int batch, int s_in, int s_out, int layers,
                       int n_dev);

/* ---- pipeline layout and search operators (paper Section 4.2, Algorithm 1; Section 4.3) --------------------------
 * Host functions, no device work.  A pipeline group is described by GPU types (the paper's vector representation):
 * count[k] GPUs of type k with memory bandwidth m_d[k], peak rate c_d[k], memory mem_bytes[k], the link inside a
 * tensor-parallel group of that type (tp_alpha[k], tp_beta[k]: same machine, same type, the paper's heuristic) and one
 * link per ordered type pair for the hop from a stage of type a to a stage of type b (pp_alpha / pp_beta, row-major
 * n_types x n_types).  All arrays are HOST arrays owned by the caller.  n_types <= 8, count[k] <= 64.
 *
 * hexgen_sched_pipeline_layout: for the given layer partition layers[n_stages], the cheapest assignment of (type,
 * degree) to every stage under the end-to-end cost of Section 4.2 (sum of Eq. 3 and Eq. 4 per stage, Eq. 5 per hop)
 * subject to the memory limit of Eq. 6 per stage, by the dynamic programme of Algorithm 1 (state: stages served, GPUs
 * used per type, type of the last stage).  GPUs may stay unused.  pow2_degrees_only != 0 restricts degrees to powers
 * of two.  Returns the cost in seconds and, when both are not NULL, the chosen type and degree per stage; +infinity
 * when no assignment fits; NaN for invalid arguments.
 *
 * hexgen_sched_merge / split / swap: the mutation operators on group vectors (split: floor / ceil halves; swap moves
 * one GPU of `type` from tau2 to tau1, in place).  hexgen_sched_repartition_layers: layer partition proportional to
 * the memory of the GPU set serving each stage, at least one layer per stage, remainder by largest fractional part.
 * These four return 1 on success, 0 for invalid arguments (outputs untouched).
 * hexgen_sched_group_can_hold: the early check on an offspring (Section 4.3): 1 when the group's total device memory
 * (sum of tau[k] * mem_bytes[k]) is at least model_bytes, else 0 (also for invalid arguments).
 */
typedef struct {
    int n_types;
    const int *count;
    const double *m_d, *c_d, *mem_bytes;
    const double *tp_alpha, *tp_beta;
    const double *pp_alpha, *pp_beta;
} hexgen_pool_t;
typedef struct {
    int hidden;
    double params_factor;
    int bytes_per_elem, batch, s_in, s_out;
} hexgen_task_t;
double hexgen_sched_pipeline_layout(const hexgen_pool_t *pool, const hexgen_task_t *task, int n_stages, const int *layers,
                                    int pow2_degrees_only, int *stage_type, int *stage_count);
int hexgen_sched_merge(int n_types, const int *tau1, const int *tau2, int *out);
int hexgen_sched_split(int n_types, const int *tau, int *out1, int *out2);
int hexgen_sched_swap(int n_types, int *tau1, int *tau2, int type);
int hexgen_sched_repartition_layers(int total_layers, int n_stages, const double *stage_mem, int *layers_out);
int hexgen_sched_group_can_hold(int n_types, const int *tau, const double *mem_bytes, double model_bytes);

/* ---- SLO attainment and the search over deployments (paper Section 5.1 "SLO attainment"; Section 4.3) -----------
 * Host functions, no device work; all arrays are HOST arrays owned by the caller.
 *
 * hexgen_slo_attainment: the share of the requests of a trace that a deployment finishes in time.  arrival[n_req]:
 * non-decreasing times >= 0 in seconds (a Poisson process in the paper's experiments); cls[n_req]: request class in
 * [0, n_classes), NULL = all class 0; latency[n_replicas][n_classes] > 0: seconds replica r needs for a request of
 * class c (the end-to-end cost of Section 4.2 of that pipeline group); deadline[n_classes].  The paper takes its task
 * simulator from another system; the queue here: requests in arrival order, none dropped, one request at a time per
 * replica, each request sent to the replica on which it finishes earliest (lowest index on ties); on time when
 * finish <= arrival + deadline.  finish_out[n_req] (may be NULL) receives the finish times.  Returns the share in
 * [0, 1]; NaN for invalid arguments (no request, unsorted or negative arrivals, a class out of range, a latency <= 0).
 *
 * hexgen_sched_draw: the search's counter-based random source: output counter + 1 of the SplitMix64 sequence started
 * at seed.
 *
 * hexgen_sched_initial_groups: the start of the search (Section 4.3 "Initialization"): weighted K-means over the GPU
 * types' rows of the hop matrices (latencies and per-byte times, each scaled by its largest entry), the number of
 * groups from the elbow of the inertia curve; every cluster of types becomes one group.  groups[n_types][n_types]
 * receives one count vector per group; returns the number of groups, 0 for invalid arguments (among them a hop
 * latency < 0 or a hop bandwidth <= 0 between types that are present) or an empty pool.
 *
 * hexgen_sched_plan_group: the pipeline a group tau (tau[k] <= count[k]) would run (Section 4.3 "Determine the
 * pipeline partitions"): for every stage count S <= min(max_stages, GPUs, layers) the even layer partition, the
 * layout of Algorithm 1, the partition proportional to the stages' memory, the layout again, the cheaper of the two;
 * over S the cheapest, fewest stages on ties.  Outputs (each may be NULL): *n_stages and layers / stage_type /
 * stage_count[max_stages].  Returns the latency in seconds, +infinity (and *n_stages = 0) when the group can run no
 * pipeline, NaN for invalid arguments.
 *
 * hexgen_sched_search: the iteration of Section 4.3 ("Put it together") for n_iter steps from the start above: pick a
 * member of the population, one of merge / split / swap and its operand groups (for swap also the GPU type, among
 * those the giving group holds) with draws 5 it .. 5 it + 4 modulo the number of choices; drop the offspring when the
 * operator does not apply, a new group fails hexgen_sched_group_can_hold for model_bytes, has more than
 * max_group_states layout states (product of tau[k] + 1) or no plan; score it by hexgen_slo_attainment over the trace
 * with the groups' plan latencies (one class); let it join the population (pop_size members at most; it replaces the
 * member of lowest score, oldest first, unless it scores lower).  A start that is not admissible is replaced by the
 * whole pool as one group.  Outputs describe the first deployment that reached the best score: *n_groups,
 * group_tau[max_groups][n_types], and (each may be NULL) group_latency[max_groups], group_n_stages[max_groups],
 * stage_layers / stage_type / stage_count[max_groups][max_stages], history[n_iter] = best score after each step.
 * Returns the best score; NaN for invalid arguments, when even the whole pool is not admissible, or when the result
 * has more than max_groups groups (outputs then untouched).
 */
typedef struct {
    int total_layers;
    double model_bytes;
    int max_stages;
    int pow2_degrees_only;
    unsigned long long seed;
    int n_iter;
    int pop_size;
    long max_group_states;
} hexgen_search_t;
double hexgen_slo_attainment(int n_req, const double *arrival, const int *cls, int n_replicas, int n_classes,
                             const double *latency, const double *deadline, double *finish_out);
unsigned long long hexgen_sched_draw(unsigned long long seed, unsigned long long counter);
int hexgen_sched_initial_groups(const hexgen_pool_t *pool, int *groups);
double hexgen_sched_plan_group(const hexgen_pool_t *pool, const hexgen_task_t *task, const int *tau, int total_layers,
                               int max_stages, int pow2_degrees_only, int *n_stages, int *layers, int *stage_type,
                               int *stage_count);
double hexgen_sched_search(const hexgen_pool_t *pool, const hexgen_task_t *task, const hexgen_search_t *cfg, int n_req,
                           const double *arrival, double deadline, int max_groups, int *n_groups, int *group_tau,
                           double *group_latency, int *group_n_stages, int *stage_layers, int *stage_type,
                           int *stage_count, double *history);

/* Bytes of device memory the stage holds for weights (after repacking), for reporting. */
int64_t hexgen_stage_weight_bytes(const hexgen_stage_t *st);

#ifdef __cplusplus
}
#endif
#endif /* HEXGEN_H */
