/*
 * emoe.h -- C ABI of the resident-expert MoE layer for AMD MI355X (gfx950).
 *
 * One MoE layer forward (a gating function that scores the experts and a set of
 * expert networks of which each token uses a few, eMoE Section 1) computed over
 * only those experts that are currently resident in GPU memory.
 * The rule that makes this the paper's layer and not the ordinary one is in
 * Section 3.2.2 (last paragraph): a token whose chosen expert is not on the
 * GPU is routed to its next-best expert that is.
 *
 * Notation: T tokens, d = d_model, f = d_ff, E experts, k experts per token,
 * S expert slots in GPU memory (a slot holds one expert's weights or is
 * empty), A = T*k assignments; assignment a = t*k + j is token t's j-th choice.
 *
 * Conventions for every entry point
 *   - "dev" pointers are device (HBM) addresses, "host" pointers are host
 *     addresses; the caller owns every buffer; the library allocates no device
 *     memory, frees nothing and keeps no state between calls, with three
 *     exceptions that the calls concerned describe: the emoe_loader object, the
 *     fixed array behind emoe_permute_static, and the number of compute units
 *     and XCDs of each device, which are looked up once and remembered.
 *   - Tensors are dense row-major.  Element type is desc->dtype: fp32, or
 *     bf16 stored as 16-bit patterns.  Pointers must be 16-byte aligned.
 *   - `stream` is a hipStream_t (NULL = the null stream).  Calls only enqueue
 *     work on it; none synchronises with the host.
 *   - Return value: EMOE_OK or a negative emoe_status.  Arguments are checked
 *     on the host before anything is enqueued; on a validation error nothing
 *     is enqueued and no output is touched.  T == 0 is a successful no-op.
 *   - Limits: 1 <= k <= S <= E <= 64; d_model and d_ff multiples of 8;
 *     (T*k + 2) * max(d_model, d_ff) <= 2^31.
 */
#ifndef EMOE_H
#define EMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    EMOE_OK = 0,
    EMOE_ERR_NULL = -1,        /* a required pointer is NULL */
    EMOE_ERR_SHAPE = -2,       /* an extent is out of range or inconsistent */
    EMOE_ERR_UNSUPPORTED = -3, /* unknown dtype / activation, E > 64, extent not a multiple of 8 */
    EMOE_ERR_RESIDENT = -4,    /* bad expert or slot id, duplicate slot, fewer than k resident experts */
    EMOE_ERR_WORKSPACE = -5,   /* workspace pointer NULL or too small */
    EMOE_ERR_DEVICE = -6       /* a HIP runtime call failed */
} emoe_status;

typedef enum { EMOE_F32 = 0, EMOE_BF16 = 1 } emoe_dtype;
typedef enum { EMOE_ACT_SWIGLU = 0, EMOE_ACT_RELU = 1 } emoe_act;

typedef struct {
    int32_t T;       /* tokens in this call                         */
    int32_t d_model; /* d                                           */
    int32_t d_ff;    /* f                                           */
    int32_t E;       /* experts the gate scores                     */
    int32_t k;       /* experts per token                           */
    int32_t S;       /* expert slots in GPU memory (see note below) */
    int32_t dtype;   /* emoe_dtype of x, weights, x_perm, y_perm, out */
    int32_t act;     /* emoe_act                                    */
} emoe_layer_desc;

/* Note on S: the row counts of the slots live on the device, so the expert FFN picks its kernels
 * (weight streaming, small or large tiles) on the host from T*k / S, the average rows per slot if
 * every slot is occupied.  Results do not depend on it, speed does: size S to the resident budget
 * (the L of Section 3.4), not to E, when far fewer experts are resident than exist. */

/* Static description of a status code; never NULL, never freed. */
const char *emoe_status_string(int status);

/* Bytes of device workspace emoe_permute and emoe_expert_ffn need for `desc`
 * (either output pointer may be NULL).  Pure host arithmetic.  The FFN workspace is
 * h [A,f] in dtype plus, for bf16 layers with more than 22 rows per slot on average,
 * 32 or 64 MiB of fp32 partial sums of output tiles cut along K.  Neither workspace
 * needs initialising, and nothing in them outlives a call except h between the two
 * passes of emoe_expert_ffn_pass.  Calls that may run at the same time (different
 * streams) need workspaces of their own. */
int emoe_workspace_bytes(const emoe_layer_desc *desc, size_t *permute_ws_bytes, size_t *ffn_ws_bytes);

/*
 * Gate and resident-restricted top-k (Section 1: the gate; Section 3.2.2: fallback
 * to the next-best resident expert; Section 3.2.2 first paragraphs: the routing
 * result of a token is a list of k expert indices).
 *   logit[t,e] = sum_i x[t,i] * w_gate[e,i] (+ gate_bias[e]), fp32 accumulation.
 *   Among experts with slot_of_expert[e] >= 0, the k largest logits in descending
 *   order (ties: lower expert index) -> topk_expert[t,0..k-1] (expert ids).
 *   topk_weight[t,j] = softmax over those k logits (fp32; sums to 1).
 * x [T,d] dev, w_gate [E,d] dev, gate_bias [E] fp32 dev or NULL,
 * slot_of_expert [E] int32 dev (-1 = not resident),
 * topk_expert [T,k] int32 dev (out), topk_weight [T,k] fp32 dev (out).
 * Precondition (not checkable on the host): at least k experts are resident;
 * emoe_load_experts never produces a map that violates it.  If it is violated
 * the outputs are unspecified, but every later call still stays in bounds.
 */
int emoe_route(const emoe_layer_desc *desc, const void *x, const void *w_gate, const float *gate_bias,
               const int32_t *slot_of_expert, int32_t *topk_expert, float *topk_weight, void *stream);

/*
 * emoe_route that also observes the experts' workload (Section 3.2.2: when memory
 * is short the experts with the larger workload are loaded first, the workload
 * being the number of tokens an expert receives).  Outputs as emoe_route; in addition, for every token,
 * expert_tokens[e] += 1 for each of the k experts the token would use if every
 * expert were resident (the k largest logits over all E experts, same tie rule).
 * expert_tokens [E] int64 dev, in/out: counts accumulate across calls (a layer
 * observes many batches between two loads); the caller zeroes it.  Integer
 * atomic adds, so the totals do not depend on execution order.
 */
int emoe_route_observe(const emoe_layer_desc *desc, const void *x, const void *w_gate, const float *gate_bias,
                       const int32_t *slot_of_expert, int32_t *topk_expert, float *topk_weight,
                       int64_t *expert_tokens, void *stream);

/*
 * Token permutation into per-slot groups (the per-expert token count is the
 * "workload" of Section 3.2.2).  Stable counting sort of the assignments
 * a = 0..A-1 by key slot_of_expert[topk_expert[a]]:
 *   slot_counts[s]  = number of assignments in slot s (0 for empty slots),
 *   slot_offsets    = exclusive prefix sum of slot_counts, length S+1,
 *   perm[r] = a     : row r of the grouped order holds assignment a,
 *   inv_perm[a] = r,
 *   x_perm[r,:]     = x[perm[r] / k, :]   (bit copy).
 * All outputs dev; ws dev, ws_bytes >= permute_ws_bytes of emoe_workspace_bytes.
 * x_perm may be NULL (then x may be NULL too): only the indices are produced, for
 * a caller that goes on with emoe_expert_ffn_gather and never needs the copy.
 */
int emoe_permute(const emoe_layer_desc *desc, const void *x, const int32_t *topk_expert,
                 const int32_t *slot_of_expert, int32_t *slot_counts, int32_t *slot_offsets, int32_t *perm,
                 int32_t *inv_perm, void *x_perm, void *ws, size_t ws_bytes, void *stream);

/*
 * emoe_permute for callers that cannot allocate device memory and have no workspace to
 * hand over: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same inputs, outputs, result and errors as emoe_permute, without `ws`: the
 * per-workgroup slot counts live in a 256 KiB array that the library keeps in every GPU's
 * memory from the moment it is loaded until the process ends.  The call allocates and frees
 * nothing.  Limit: ceil(T*k / 1024) * S <= 65536, else EMOE_ERR_WORKSPACE (nothing is
 * enqueued).  All calls on one GPU share that GPU's array: calls that may overlap on one
 * GPU (different streams, or threads) race; calls on one stream, one after the other, do
 * not, and nothing needs clearing between them.  The first call on a device looks the
 * array's address up (a host-side query, no stream work); make it outside graph capture.
 */
int emoe_permute_static(const emoe_layer_desc *desc, const void *x, const int32_t *topk_expert,
                        const int32_t *slot_of_expert, int32_t *slot_counts, int32_t *slot_offsets, int32_t *perm,
                        int32_t *inv_perm, void *x_perm, void *stream);

/*
 * Expert FFN over the grouped rows, only for slots that received rows (Section 5.1
 * attributes the method's latency gain to exactly this: with fewer experts there
 * is less to compute and less to read from GPU memory).  For slot s and rows r in [slot_offsets[s], slot_offsets[s+1]):
 *   SwiGLU: h = silu(x_perm[r] W1_s^T) * (x_perm[r] W3_s^T),  y_perm[r] = h W2_s^T
 *   ReLU  : h = max(x_perm[r] W1_s^T, 0),                      y_perm[r] = h W2_s^T
 * Products accumulate in fp32; h and y_perm are rounded once to dtype.
 * x_perm [A,d] dev; slot_offsets [S+1] dev; w1_slots, w3_slots [S,f,d] dev
 * (w3_slots must be NULL for ReLU and non-NULL for SwiGLU); w2_slots [S,d,f] dev;
 * y_perm [A,d] dev (out); ws dev, ws_bytes >= ffn_ws_bytes.
 */
int emoe_expert_ffn(const emoe_layer_desc *desc, const void *x_perm, const int32_t *slot_offsets,
                    const void *w1_slots, const void *w3_slots, const void *w2_slots, void *y_perm, void *ws,
                    size_t ws_bytes, void *stream);

/*
 * One half of emoe_expert_ffn, with the same arguments and checks: pass 1 computes
 * h (into ws) from x_perm, pass 2 computes y_perm from the h that pass 1 left in ws.
 * Calling pass 1 then pass 2 on one stream is emoe_expert_ffn.  Exists so that each of the two
 * grouped products can be timed and profiled on its own.  Any other `pass`: EMOE_ERR_SHAPE.
 */
int emoe_expert_ffn_pass(const emoe_layer_desc *desc, int32_t pass, const void *x_perm,
                         const int32_t *slot_offsets, const void *w1_slots, const void *w3_slots,
                         const void *w2_slots, void *y_perm, void *ws, size_t ws_bytes, void *stream);

/*
 * emoe_expert_ffn with the row gather folded into the first product's operand
 * load: grouped row r is read as x[perm[r] / k, :] straight from the token matrix,
 * so x_perm is neither written nor read (it is the dominant glue traffic of a
 * layer with many small experts).  Same result as emoe_permute's x_perm followed
 * by emoe_expert_ffn, bit for bit.  x [T,d] dev, perm [A] dev (from emoe_permute);
 * everything else as emoe_expert_ffn.  emoe_expert_ffn_gather_pass: its two
 * halves, as emoe_expert_ffn_pass.
 */
int emoe_expert_ffn_gather(const emoe_layer_desc *desc, const void *x, const int32_t *perm,
                           const int32_t *slot_offsets, const void *w1_slots, const void *w3_slots,
                           const void *w2_slots, void *y_perm, void *ws, size_t ws_bytes, void *stream);
int emoe_expert_ffn_gather_pass(const emoe_layer_desc *desc, int32_t pass, const void *x, const int32_t *perm,
                                const int32_t *slot_offsets, const void *w1_slots, const void *w3_slots,
                                const void *w2_slots, void *y_perm, void *ws, size_t ws_bytes, void *stream);

/*
 * Gate-weighted combine back to token order (Section 1):
 *   out[t,:] = sum_{j<k} topk_weight[t,j] * y_perm[inv_perm[t*k+j], :], j ascending,
 * fp32 accumulation, one rounding to dtype.  out [T,d] dev.
 */
int emoe_combine(const emoe_layer_desc *desc, const void *y_perm, const int32_t *inv_perm,
                 const float *topk_weight, void *out, void *stream);

/*
 * emoe_expert_ffn_gather followed by emoe_combine as one call, with the combine folded into the
 * second product where that costs nothing (Section 5.1: fewer global-memory reads): in a layer
 * with one expert per token (k = 1) the gate weight is exactly 1 and the combine only undoes the
 * row permutation, so the second product stores grouped row r straight into out[perm[r], :];
 * y_perm is then neither written nor read (it may be NULL) and one launch is saved.  For k > 1 a
 * token's k rows come from different output tiles and the call is the two calls as they are.
 * The result in `out` is that of the two calls bit for bit.  Arguments as in the two calls.
 */
int emoe_expert_ffn_gather_combine(const emoe_layer_desc *desc, const void *x, const int32_t *perm,
                                   const int32_t *inv_perm, const int32_t *slot_offsets, const void *w1_slots,
                                   const void *w3_slots, const void *w2_slots, const float *topk_weight, void *y_perm,
                                   void *out, void *ws, size_t ws_bytes, void *stream);

/*
 * The whole layer (Section 1: gate plus experts, here over the resident
 * experts only, Section 3.2.2): emoe_route, emoe_permute (indices only) and
 * emoe_expert_ffn_gather_combine enqueued in this order on `stream`, with the same arguments,
 * results and errors as the single calls; nothing else is done and nothing is allocated (with
 * k = 1 y_perm stays unwritten, see emoe_expert_ffn_gather_combine).  All the intermediate
 * results are caller buffers as in the single calls (x_perm is not needed: the FFN reads the
 * token rows through perm).  Validation of all arguments happens before the first launch, so an
 * error leaves every output untouched.
 */
int emoe_layer_forward(const emoe_layer_desc *desc, const void *x, const void *w_gate, const float *gate_bias,
                       const int32_t *slot_of_expert, const void *w1_slots, const void *w3_slots,
                       const void *w2_slots, int32_t *topk_expert, float *topk_weight, int32_t *slot_counts,
                       int32_t *slot_offsets, int32_t *perm, int32_t *inv_perm, void *y_perm, void *out,
                       void *permute_ws, size_t permute_ws_bytes, void *ffn_ws, size_t ffn_ws_bytes, void *stream);

/*
 * Change the resident set (Section 3.2.2: predicted experts not yet on the GPU are
 * loaded, the others leave; Section 4: loads are asynchronous host-to-device copies,
 * the layer waits on an event recorded after its load so it never sees stale
 * weights, and loads are issued one after the other so the host link is not
 * oversubscribed).
 *
 * For i in 0..n-1 (in this order): slot slot_ids[i] receives expert expert_ids[i];
 * expert_ids[i] == -1 only empties the slot.  An expert already resident in
 * another slot moves (its old slot becomes empty).  Whatever the slot held before
 * is dropped; the host keeps the master copy of every expert, nothing is copied back.
 *
 * host_w1/w3/w2: host arrays of E host pointers to each expert's weights in
 * canonical layout W1 [f,d], W3 [f,d], W2 [d,f]; only entries named in expert_ids
 * are read; they must stay valid and unchanged until done_event (or the stream)
 * completes, and should be pinned for the copy to be asynchronous.  host_w3 may
 * be NULL for ReLU.
 * w1_slots/w3_slots/w2_slots: dev slot buffers [S,f,d], [S,f,d], [S,d,f].
 * slot_of_expert [E] dev, expert_of_slot [S] dev: the device maps (out).
 * expert_of_slot_host [S] host (in/out): the caller's mirror of expert_of_slot
 * (-1 = empty); read to validate the change, updated on success.
 *
 * Order on side_stream: wait wait_event (if not NULL: "no layer forward still
 * reads these slots") -> copies in list order -> both device maps rewritten ->
 * record done_event (if not NULL).  A forward that must see the new experts
 * waits on done_event first.
 * Errors found by validation (nothing enqueued, mirror untouched): EMOE_ERR_RESIDENT
 * for ids out of range, a slot named twice, an expert named twice, or a resulting
 * map with fewer than k resident experts; EMOE_ERR_NULL / _SHAPE as everywhere.
 * EMOE_ERR_DEVICE (a HIP call failed while enqueueing) is different: copies
 * issued before the failure stay enqueued, the device maps and done_event may
 * not have been written and the mirror is left as it was, so the named slots
 * and both device maps are undefined until the next successful call that names
 * the same slots; the caller should treat those slots as empty.
 */
int emoe_load_experts(const emoe_layer_desc *desc, int32_t n, const int32_t *expert_ids, const int32_t *slot_ids,
                      const void *const *host_w1, const void *const *host_w3, const void *const *host_w2,
                      void *w1_slots, void *w3_slots, void *w2_slots, int32_t *slot_of_expert,
                      int32_t *expert_of_slot, int32_t *expert_of_slot_host, void *side_stream, void *wait_event,
                      void *done_event);

/*
 * Choice of the resident experts of one layer (Section 3.4).  Host-only helpers:
 * every pointer is host memory, nothing is enqueued, no GPU is needed.
 *
 * emoe_expected_tokens: Eq. 2.  For every task type t,
 *   N_i = (sum of W_j over the running requests j of type t + T_t * W_o[t]) * s[t] * f[t,i],
 * T_t = number of running requests of type t; expected[i] = sum over t of N_i,
 * accumulated in ascending t in double precision.
 *   freq [n_tasks,E] predicted routing frequencies f, request_task [n_requests]
 *   (0..n_tasks-1), request_tokens [n_requests] = W_j >= 0, w_out [n_tasks] = W_o,
 *   sensitive [n_tasks] = s (0 or nonzero), expected [E] out.
 *
 * emoe_select_experts: the L experts with the largest expected[], in descending
 * order (equal values: lower index first) -> selected [L].  1 <= L <= E.
 *
 * emoe_plan_load: Section 3.2.2, last paragraph.  Compares the selection with the
 * residents (expert_of_slot_host [S], -1 = empty) and writes the list that
 * emoe_load_experts takes: selected experts that are not resident, in the order
 * of `selected` (higher workload first), each into the lowest slot that is empty
 * or holds an unselected expert; then an entry (-1, slot) for every slot still
 * holding an unselected expert.  Resident selected experts are not moved.
 * expert_ids, slot_ids: out, capacity S; *n = entries written (0 = nothing to
 * do).  The map is not modified (emoe_load_experts does that).
 * EMOE_ERR_RESIDENT: L > S, L < k, an id out of range or repeated.
 */
int emoe_expected_tokens(int32_t E, int32_t n_tasks, const double *freq, int32_t n_requests,
                         const int32_t *request_task, const int64_t *request_tokens, const double *w_out,
                         const int32_t *sensitive, double *expected);
int emoe_select_experts(int32_t E, const double *expected, int32_t L, int32_t *selected);
int emoe_plan_load(int32_t E, int32_t S, int32_t k, const int32_t *expert_of_slot_host, int32_t L,
                   const int32_t *selected, int32_t *expert_ids, int32_t *slot_ids, int32_t *n);

/*
 * Periodic loading for a stack of MoE layers (Section 3.3: requests are numbered
 * 0, 1, 2, ...; for the first one all experts are loaded, for every p-th one the
 * predictor is invoked and only the predicted experts are loaded, all others
 * reuse the residents.  Section 4: a layer's load and the layer's computation
 * are ordered against each other, and layer i+1's load begins only after layer
 * i's has finished, so that loads never compete for the host link).
 *
 * emoe_prompt_action: the rule alone (host only, no GPU needed).  Returns
 * EMOE_PROMPT_LOAD_ALL for index 0 if all experts fit the slots (S == E in every
 * layer; otherwise index 0 needs a prediction like a p-th prompt),
 * EMOE_PROMPT_PREDICT if index % period == 0, else EMOE_PROMPT_REUSE; negative
 * emoe_status on a bad argument.
 *
 * emoe_loader: the object that applies it.  It owns one side stream (default
 * priority), two events per layer and the host mirrors of the slot maps, which
 * start empty; everything in emoe_loader_layer stays the caller's and must
 * outlive the loader (host_w*: arrays [E] of pinned host pointers, as for
 * emoe_load_experts; desc.T is ignored).  Not thread safe.
 *   create        EMOE_ERR_DEVICE if stream or events cannot be created.
 *   next_prompt   numbers the prompt and reports its action; for LOAD_ALL it has
 *                 already enqueued the loads (expert e into slot e, layer after
 *                 layer).  For PREDICT the caller obtains the prediction and
 *                 calls update before the prompt's first layer.
 *   update        selected[i] = L[i] expert ids of layer i in descending
 *                 workload order.  Plans every layer (emoe_plan_load) and then
 *                 enqueues the changed layers' loads on the side stream in
 *                 layer order; each waits until that layer's last forward has
 *                 released its slots.  All layers are planned and validated
 *                 before the first is enqueued, so an argument error enqueues
 *                 nothing and changes nothing.  EMOE_ERR_DEVICE from layer i
 *                 leaves layers before i loaded and recorded in their mirrors
 *                 (they are consistent and usable), layer i as described for
 *                 emoe_load_experts, and later layers untouched.
 *   layer_begin   call before layer i's forward: makes compute_stream wait for
 *                 the layer's pending load, if any (no stale weights).
 *   layer_end     call after layer i's forward: marks on compute_stream the
 *                 point after which the layer's slots may be overwritten.
 *   layer_ready   does not block: *ready = 1 if every load enqueued for layer i so
 *                 far has finished on the GPU (a forward of it would not wait), else 0.
 *   residents     copies layer i's host mirror expert_of_slot [S].
 *   synchronize   blocks the host until every enqueued load has finished.
 *   destroy       synchronizes the side stream, then frees the object.
 */
enum { EMOE_PROMPT_REUSE = 0, EMOE_PROMPT_LOAD_ALL = 1, EMOE_PROMPT_PREDICT = 2 };
typedef struct emoe_loader emoe_loader;
typedef struct {
    emoe_layer_desc desc;
    const void *const *host_w1, *const *host_w3, *const *host_w2;
    void *w1_slots, *w3_slots, *w2_slots;
    int32_t *slot_of_expert, *expert_of_slot;
} emoe_loader_layer;

int emoe_prompt_action(int64_t prompt_index, int32_t period, int32_t all_experts_fit);
int emoe_loader_create(int32_t n_layers, const emoe_loader_layer *layers, int32_t period, emoe_loader **out);
int emoe_loader_destroy(emoe_loader *loader);
int emoe_loader_next_prompt(emoe_loader *loader, int64_t *prompt_index, int32_t *action);
int emoe_loader_update(emoe_loader *loader, const int32_t *const *selected, const int32_t *L);
int emoe_loader_layer_begin(emoe_loader *loader, int32_t layer, void *compute_stream);
int emoe_loader_layer_end(emoe_loader *loader, int32_t layer, void *compute_stream);
int emoe_loader_layer_ready(const emoe_loader *loader, int32_t layer, int32_t *ready);
int emoe_loader_residents(const emoe_loader *loader, int32_t layer, int32_t *expert_of_slot_host);
int emoe_loader_synchronize(emoe_loader *loader);

/*
 * Request scheduler (Section 3.5).  Host-only, no GPU needed.
 *
 * emoe_request: input_tokens = W of the request; slo = its latency SLO;
 * first_token_slo = how soon its first token is due (the stringency the waiting
 * queue is ordered by); run_time = r_i so far; g_remaining = G_i, tokens it
 * still has to generate (the task's profiled length when scheduled); g_initial
 * = that profiled length; delta_e = expert loading latency that scheduling this
 * request causes (profiled; 0 for a task no layer is sensitive to).
 *
 * emoe_expected_latency: Eq. 3 for running request i,
 *   t_i = dE + (W + n_i * G_i) * c + r_i,
 * n_i = running requests other than i with more tokens left than i; dE and W
 * from new_request, or 0 if new_request is NULL (the latency as things stand).
 *
 * emoe_schedule: Algorithm 1.  The waiting requests are tried in ascending
 * first_token_slo (equal values in queue order).  A request is admitted if its
 * input tokens plus those held by the scheduled requests stay below t_max, and
 * every running request whose expected latency is below its SLO now keeps it
 * below its SLO with the new request (Eq. 3).  An admitted request joins the
 * running ones (run_time 0) for the candidates after it.  admitted [n_waiting]
 * out: indices into `waiting` in admission order; *n_admitted their number.
 *
 * emoe_generation_tick: after one iteration of token generation G_i is
 * decremented; if it reaches 0 and the request has not completed it is reset
 * to reset_fraction (the paper's example: 0.05) of g_initial, at least 1.
 */
typedef struct {
    int32_t input_tokens;
    int32_t g_remaining;
    int32_t g_initial;
    int32_t reserved;
    double slo;
    double first_token_slo;
    double run_time;
    double delta_e;
} emoe_request;

int emoe_expected_latency(int32_t n_running, const emoe_request *running, int32_t i, double c,
                          const emoe_request *new_request, double *latency);
int emoe_schedule(int32_t n_waiting, const emoe_request *waiting, int32_t n_scheduled,
                  const emoe_request *scheduled, int64_t t_max, double c, int32_t *admitted, int32_t *n_admitted);
int emoe_generation_tick(emoe_request *request, int32_t completed, double reset_fraction);

/*
 * Measurement aids (no step of the layer; for the benchmark's measured ceilings beside the
 * datasheet peaks).  Both only enqueue one kernel on `stream`; the caller times it.
 *
 * emoe_measure_mfma_loop: `workgroups` workgroups of four wavefronts each copy a 256 x 64 tile
 * of a and of b (dev, bf16, a_elems / b_elems elements, at least 16384 each; pass the workload's
 * own token rows and weights so that the operand values are the GEMM's) into LDS once and then
 * issue `iters` rounds of 4 x 16 matrix instructions (v_mfma_f32_32x32x16_bf16, 4 x 4 blocks per
 * wavefront as in the tiled FFN kernel) with no global memory traffic; lds_reads != 0 adds the
 * GEMM's LDS fragment reads (8 per 16 matrix instructions).  sink: dev, workgroups * 256 floats
 * (out, meaningless sums).  *flop (host, may be NULL) = workgroups * 4 * iters * 64 * 32768.
 *
 * emoe_measure_read_stream: grid-stride read of src (dev, `bytes` a multiple of 32768) with
 * 16-byte loads, eight in flight per lane, nothing written.  sink: dev, 16 bytes.
 *
 * emoe_measure_copy_stream: plain copy of `bytes` (a multiple of 16) from src to dst (dev, not
 * overlapping): reads and writes exactly `bytes`, the kernel of known traffic by which the
 * readings of HBM traffic counters in the same profiler run are scaled.
 */
int emoe_measure_mfma_loop(const void *a, size_t a_elems, const void *b, size_t b_elems, int32_t lds_reads,
                           int32_t workgroups, int32_t iters, float *sink, double *flop, void *stream);
int emoe_measure_read_stream(const void *src, size_t bytes, int32_t workgroups, void *sink, void *stream);
int emoe_measure_copy_stream(const void *src, void *dst, size_t bytes, int32_t workgroups, void *stream);

/*
 * emoe_measure_scatter_combine: emoe_combine computed the way a second product with the combine
 * folded into its epilogue would have to compute it for k > 1: an fp32 image of the output is
 * cleared, every grouped row is added into its token's row with atomics (weighted by its gate
 * weight), and the image is converted to bf16.  Same inputs as emoe_combine except that rows are
 * found through perm [A] (grouped row -> assignment) and `image` [T,d] fp32 dev is scratch.  bf16
 * layers only.  The sum's order is that of the atomics: for k = 2 the result is reproducible,
 * beyond that it is not.  Exists to measure the cost of that design against emoe_combine.
 */
int emoe_measure_scatter_combine(const emoe_layer_desc *desc, const void *y_perm, const int32_t *perm,
                                 const float *topk_weight, float *image, void *out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* EMOE_H */
