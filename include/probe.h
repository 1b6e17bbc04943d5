/*
 * probe.h - C ABI of libprobe: one GPU's share of an expert-parallel MoE layer on MI355X
 * (gfx950), after PROBE (arxiv 2602.00509).
 *
 * The five calls are the steps of the layer's main track (Sec. 4.1 of the paper) that run
 * on one GPU between the two all-to-all exchanges, plus the lookahead predictor of the
 * auxiliary track (Sec. 4.2):
 *
 *   probe_route_topk    router of layer L: logits W_L h + b_L, softmax, k largest
 *   probe_predict_topk  gate-initialised lookahead predictor (Eq. 7, frozen prior term);
 *                       probe_predict_topk_residual adds the trainable residual MLP of Eq. 7
 *   probe_plan_greedy   the greedy planner of Sec. 4.3 (Algorithm 1): predicted workload -> plan
 *   probe_permute       group (token, top-k position) pairs by the expert replica that the
 *                       balance plan (placement P, assignment A; Sec. 3.1, Sec. 4.3) gives them
 *   probe_grouped_ffn   grouped SwiGLU expert FFN over native + replicated experts
 *                       (E_r U Delta_r, Sec. 3.2)
 *   probe_combine       gate-weighted sum of a token's expert outputs (local part of the
 *                       combine step)
 *
 * Variants of these: probe_pack_gate and the *_packed router / predictor calls (the gate's bf16 planes
 * made once instead of per call), probe_permute_static (no workspace, for callers that cannot
 * allocate), probe_route_predict_topk (router and next layer's predictor in one pass over
 * the hidden states), probe_route_grouped (a model's group-limited gate in place of the plain
 * top-k), probe_grouped_ffn_gather (activation rows gathered on load, no permuted copy),
 * probe_combine_shared (adds a shared expert's output), probe_plan_dispatch (the plan as the source
 * rank applies it to its own tokens ahead of the dispatch exchange), and probe_predictor_metrics
 * (top-k accuracy and distillation cross-entropy of a predictor, evaluation only).
 *
 * Conventions for every call
 *   - Every pointer marked "device" is caller-owned device memory; the library never
 *     allocates, frees, synchronises or copies to the host inside these calls.  Sizes that
 *     depend on the data (rows per slot, number of local rows) exist only in device memory,
 *     so a sequence of calls can be recorded in a HIP graph (Sec. 2.3: no host-device
 *     synchronisation on the serving path).
 *   - `stream` is the caller's hipStream_t passed as void* (NULL = the default stream).
 *   - bf16 tensors are raw 16-bit patterns, row-major, innermost dimension contiguous.
 *   - Device pointers must be 16-byte aligned unless stated otherwise.
 *   - Return value: PROBE_OK or a negative error code.  Arguments are validated on the host
 *     before anything is launched; a failing call launches nothing.
 *     probe_last_error_string() describes the last failure on the calling thread.
 *   - `workspace` is device scratch of at least probe_<name>_workspace_bytes(...) bytes; its
 *     contents are undefined on entry and on return.  Calls that share a workspace must be
 *     ordered on one stream.
 *
 * Vocabulary: T tokens, H hidden size, E routed experts, k experts per token, F expert FFN
 * width, S weight slots on this GPU (one expert copy each), pair p = t*k + s (token t,
 * top-k position s), N = T*k pairs.
 */
#ifndef PROBE_H_
#define PROBE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PROBE_OK            0
#define PROBE_EINVAL       -1  /* null pointer, non-positive dimension, k > E, bad plan size */
#define PROBE_EUNSUPPORTED -2  /* shape outside the kernels' limits (see each call)          */
#define PROBE_EALIGN       -3  /* a device pointer is not 16-byte aligned                     */
#define PROBE_EWORKSPACE   -4  /* workspace is NULL or too small                              */
#define PROBE_EHIP         -5  /* the HIP runtime rejected a launch                           */

/* Limits of this build. */
#define PROBE_MAX_EXPERTS 256  /* E                         */
#define PROBE_MAX_TOPK      8  /* k                         */
#define PROBE_MAX_SLOTS  1024  /* S                         */
#define PROBE_MAX_RESIDUAL_WIDTH 1024 /* D of the predictor's residual MLP */
#define PROBE_MAX_GROUPS   16  /* n_group of the group-limited gate */

/* Text of the last error raised on the calling thread ("" if none). Host pointer, owned by
 * the library, valid until the next failing call on the same thread. */
const char* probe_last_error_string(void);

/* Library version, e.g. "0.1". Host pointer, static storage. */
const char* probe_version(void);

/* ------------------------------------------------------------------ route / predict ---
 *
 * Router of Sec. 4.2: l[t,e] = sum_h x[t,h] * w_gate[e,h] + bias[g(t),e];
 * p = softmax of l over all E experts; the k experts with the largest logits in descending
 * order (exact ties: lower expert index first); topk_w[t,s] = p[t, topk_idx[t,s]], divided
 * by their sum over s when `renormalize` is non-zero; expert_counts[e] = number of pairs
 * routed to e (n_e of Table 1, sum_e n_e = T*k).
 *
 *   x_bf16         device, bf16 [T,H]
 *   w_gate         device, fp32 [E,H]
 *   bias           device, fp32 [bias_groups,E], or NULL for no bias
 *   bias_groups    G >= 1; token t uses bias row min(t / tokens_per_group, G-1).  G = 1 is
 *                  the paper's single b_L; G > 1 lets one call carry a hot set that moves
 *                  between chunks of tokens.
 *   topk_idx       device, int32 [T,k]       (out)
 *   topk_w         device, fp32  [T,k]       (out)
 *   probs          device, fp32  [T,E] or NULL (out, full softmax)
 *   expert_counts  device, int32 [E] or NULL (out)
 *
 * Arithmetic: x is bf16 exactly, w_gate is used at full fp32 precision (three bf16 planes
 * on the matrix cores), accumulation in fp32.
 * Limits: 1 <= k <= 8, k <= E <= 256, H % 8 == 0, T >= 0 (T = 0 writes only zero counts).
 */
size_t probe_route_topk_workspace_bytes(int T, int H, int E, int k);

int probe_route_topk(const void* x_bf16, const float* w_gate, const float* bias,
                     int bias_groups, int tokens_per_group, int T, int H, int E, int k,
                     int renormalize, int32_t* topk_idx, float* topk_w, float* probs,
                     int32_t* expert_counts, void* workspace, size_t workspace_bytes,
                     void* stream);

/* The router with the gate of a model that limits a token to a few groups of experts.  The paper
 * (Sec. 1) targets such models and leaves each model's gate as published; this is the gate of the
 * DeepSeek-V3 technical report (Sec. 2.1.2: sigmoid affinities, gating values normalised over the
 * chosen experts, a balancing bias that enters the selection only) with its node-limited routing in
 * the form the released model configures.  Per token:
 *   l_e = logits as in probe_route_topk (bias is the paper's b_L, added to the logits)
 *   s_e = sigmoid(l_e) (PROBE_SCORE_SIGMOID) or softmax(l)_e (PROBE_SCORE_SOFTMAX)
 *   c_e = s_e + select_bias[e]                      selection score (select_bias may be NULL)
 *   group j = experts j*E/n_group .. (j+1)*E/n_group - 1; its score is the sum of its group_top
 *             largest c_e; the topk_group groups with the largest scores are allowed
 *   topk_idx = the k allowed experts with the largest c_e, descending
 *   topk_w   = s_e of the chosen experts (without select_bias), divided by their sum when
 *              renormalize is non-zero, times routed_scale
 * Equal scores go to the lower index (groups and experts alike).  n_group = topk_group = 1 with
 * softmax scores is probe_route_topk.  All decisions are taken in fp32.
 *   select_bias    device, fp32 [E] or NULL
 *   gating         host pointer, read during the call
 *   scores         device, fp32 [T,E] or NULL (out, s_e)
 * Other arguments, workspace, arithmetic of the logits and limits as probe_route_topk; in addition
 * n_group <= 16 and divides E, 1 <= topk_group <= n_group, 1 <= group_top <= E / n_group,
 * k <= topk_group * E / n_group.
 */
#define PROBE_SCORE_SOFTMAX 0
#define PROBE_SCORE_SIGMOID 1

typedef struct probe_gating {
  int32_t scoring;     /* PROBE_SCORE_SOFTMAX or PROBE_SCORE_SIGMOID */
  int32_t n_group;     /* groups of E / n_group consecutive experts */
  int32_t topk_group;  /* groups a token may use */
  int32_t group_top;   /* how many of a group's largest selection scores make up its score */
  int32_t renormalize; /* divide the gating values by their sum */
  float routed_scale;  /* factor on the gating values */
} probe_gating;

size_t probe_route_grouped_workspace_bytes(int T, int H, int E, int k);

int probe_route_grouped(const void* x_bf16, const float* w_gate, const float* bias, int bias_groups,
                        int tokens_per_group, const float* select_bias, const probe_gating* gating,
                        int T, int H, int E, int k, int32_t* topk_idx, float* topk_w, float* scores,
                        int32_t* expert_counts, void* workspace, size_t workspace_bytes,
                        void* stream);

/* Gate-initialised lookahead predictor (Eq. 7) with its trainable residual at the zero
 * initialisation the paper prescribes: the cloned router (w_gate_next, bias_next) of layer L
 * applied to the hidden states h_prev of layer L-1.  Same arguments, limits and arithmetic
 * as probe_route_topk; pred_counts is the predicted per-expert workload n-hat that the
 * planner consumes (Sec. 4.3).  The prediction never changes dispatch. */
size_t probe_predict_topk_workspace_bytes(int T, int H, int E, int k);

int probe_predict_topk(const void* h_prev_bf16, const float* w_gate_next,
                       const float* bias_next, int bias_groups, int tokens_per_group, int T,
                       int H, int E, int k, int renormalize, int32_t* pred_idx, float* pred_w,
                       float* probs, int32_t* pred_counts, void* workspace,
                       size_t workspace_bytes, void* stream);

/* Eq. 7 in full: pred_logits = W_L h + b_L + W2_hat silu(W1_hat h), silu(u) = u / (1 + exp(-u)),
 * then softmax / top-k / counts exactly as above.  The paper fixes neither the hidden width D of
 * the residual MLP nor how its weights are stored; here
 *   w1_hat_bf16  device, bf16 [D,H]  (first layer, no bias)
 *   w2_hat       device, fp32 [E,D]  (second layer, no bias; all zeros = probe_predict_topk)
 * u is accumulated in fp32 from exact bf16 x bf16 products on the matrix cores, silu and the second
 * layer run in fp32.  Other arguments and limits as probe_route_topk; D % 8 == 0, D <= 1024.
 */
size_t probe_predict_topk_residual_workspace_bytes(int T, int H, int E, int k, int D);

int probe_predict_topk_residual(const void* h_prev_bf16, const float* w_gate_next,
                                const float* bias_next, int bias_groups, int tokens_per_group,
                                const void* w1_hat_bf16, const float* w2_hat, int D, int T, int H,
                                int E, int k, int renormalize, int32_t* pred_idx, float* pred_w,
                                float* probs, int32_t* pred_counts, void* workspace,
                                size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------- permute ---
 *
 * The balance plan as this GPU sees it (Sec. 3.1: n_{e,r} with sum_r n_{e,r} = n_e; Sec. 4.3:
 * n_{e,r} > 0 only where P_{r,e} = 1).  Expert e owns replicas rep_off[e] .. rep_off[e+1]-1.
 * Replica i lives in local weight slot rep_slot[i] in [0,S), or on another GPU (-1), and
 * receives rep_weight[i] out of every P_e = sum of e's weights consecutive arrivals
 * (weighted round-robin in pair order; P_e >= 1, weights >= 0).  A weight slot holds one copy of
 * one expert: no slot id may appear twice in rep_slot (the rows of a slot are then the arrivals of
 * one replica, which is what lets a pair's row be computed without atomics); a plan that breaks
 * this gives unspecified rows for the slots concerned.  The struct itself is host memory; the
 * three arrays are device memory, int32.
 */
typedef struct {
  const int32_t* rep_off;    /* device [E+1] */
  const int32_t* rep_slot;   /* device [R], R = rep_off[E] */
  const int32_t* rep_weight; /* device [R] */
  int32_t num_slots;         /* S */
} probe_plan;

/*
 * Pairs are visited in ascending p = t*k + s.  The j-th arrival (from 0) of expert e goes to
 * the first of its replicas whose cumulative weight exceeds j mod P_e.  Pairs sent to a local
 * slot are grouped by slot, ascending p inside a slot; rows are the groups in slot order.
 *
 *   topk_idx      device, int32 [T,k], values in [0,E)
 *   x_bf16        device, bf16 [T,H]
 *   slot_counts   device, int32 [S]    (out) rows per slot
 *   slot_offsets  device, int32 [S+1]  (out) exclusive prefix sum; [S] = n_local
 *   row_pair      device, int32 [T*k]  (out) pair of each row; entries >= n_local are -1
 *   pair_row      device, int32 [T,k]  (out) row of each pair, -1 = computed on another GPU
 *   xp_bf16       device, bf16 [T*k,H] (out) xp[row] = x[row_pair[row] / k]; rows >= n_local
 *                 are not written.  May be NULL: then no row is copied (for callers that gather
 *                 the rows on load, probe_grouped_ffn_gather) and x_bf16 is not read
 *   n_local       device, int32 [1]    (out)
 *
 * Integer outputs and row copies are exact.  Limits: E <= 256, k <= 8, S <= 1024, H % 8 == 0,
 * T*k < 2^31.  An out-of-range expert id or slot id is undefined behaviour.
 */
size_t probe_permute_workspace_bytes(int T, int E, int k, int S);

int probe_permute(const int32_t* topk_idx, const probe_plan* plan, const void* x_bf16, int T,
                  int H, int E, int k, int32_t* slot_counts, int32_t* slot_offsets,
                  int32_t* row_pair, int32_t* pair_row, void* xp_bf16, int32_t* n_local,
                  void* workspace, size_t workspace_bytes, void* stream);

/* probe_permute for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc) and have no workspace to hand over: the same
 * arguments without `workspace`.  The block histograms that probe_permute keeps in its workspace live
 * in a static device array of PROBE_PERMUTE_STATIC_SCRATCH_BYTES inside the library instead; every GPU
 * the library runs on holds its own copy until the process ends.  The call allocates and frees nothing.
 * Outputs are those of probe_permute, bit for bit.
 * Limit: probe_permute_workspace_bytes(T, E, k, S) <= PROBE_PERMUTE_STATIC_SCRATCH_BYTES, i.e. at most
 * probe_permute_static_max_pairs(E) pairs (262144 at E = 256); larger batches return
 * PROBE_EUNSUPPORTED and launch nothing.  Batches of at most 1024 pairs do not touch the array.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different
 * streams, or graphs replayed concurrently) race on it and give unspecified index outputs; calls ordered
 * on one stream are safe, the array carries nothing from one call to the next.  The first call on a
 * device looks the array's address up (no allocation); make that first call outside a graph capture.
 */
#define PROBE_PERMUTE_STATIC_SCRATCH_BYTES (256 * 1024)

size_t probe_permute_static_max_pairs(int E);

int probe_permute_static(const int32_t* topk_idx, const probe_plan* plan, const void* x_bf16, int T,
                         int H, int E, int k, int32_t* slot_counts, int32_t* slot_offsets,
                         int32_t* row_pair, int32_t* pair_row, void* xp_bf16, int32_t* n_local,
                         void* stream);

/* ------------------------------------------------------------------------ grouped FFN ---
 *
 * Grouped GEMM over the experts resident on this GPU (Sec. 3.2, T_comp over E_r U Delta_r).
 * For every slot s and every row r in [slot_offsets[s], slot_offsets[s+1]):
 *     a = W1_s xp[r],  c = W3_s xp[r],  h = silu(a) * c,  y[r] = W2_s h
 *
 *   xp_bf16       device, bf16 [max_rows,H]
 *   slot_offsets  device, int32 [S+1], non-decreasing, slot_offsets[S] <= max_rows
 *   w13_ptrs      device array [S] of device pointers, each bf16 [2F,H]: rows 0..F-1 are W1
 *                 (gate projection), rows F..2F-1 are W3 (up projection)
 *   w2_ptrs       device array [S] of device pointers, each bf16 [H,F]
 *   max_rows      capacity of xp / y in rows (T*k); sizes the launch, not the work
 *   y_bf16        device, bf16 [max_rows,H] (out); rows >= slot_offsets[S] are not written
 *
 * bf16 inputs, fp32 accumulation on the matrix cores, h rounded to bf16 between the two
 * GEMMs, bf16 output.  An empty slot does no work and its weights are not read.
 * Limits: H % 64 == 0, F % 64 == 0, H and F at most 2^21, 1 <= S <= 1024, one expert's w13 below
 * 2 GiB.
 */
size_t probe_grouped_ffn_workspace_bytes(int S, int H, int F, int max_rows);

int probe_grouped_ffn(const void* xp_bf16, const int32_t* slot_offsets,
                      const void* const* w13_ptrs, const void* const* w2_ptrs, int S, int H,
                      int F, int max_rows, void* y_bf16, void* workspace,
                      size_t workspace_bytes, void* stream);

/* The same FFN with its activation rows gathered on load: row r of the row space is
 * x[row_pair[r] / k], read straight from the token rows while the first GEMM fills its tiles, so the
 * permuted copy xp is never written or read (call probe_permute with xp_bf16 = NULL: it then
 * produces its index outputs only).  Output and arithmetic are those of probe_grouped_ffn on
 * xp = gather(x).
 *   x_bf16    device, bf16 [T,H]
 *   row_pair  device, int32 [max_rows] as written by probe_permute (entries >= n_local are not read)
 * Additional limit: x below 2 GiB.
 */
int probe_grouped_ffn_gather(const void* x_bf16, const int32_t* row_pair, int T, int k,
                             const int32_t* slot_offsets, const void* const* w13_ptrs,
                             const void* const* w2_ptrs, int S, int H, int F, int max_rows,
                             void* y_bf16, void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------- combine ---
 *
 * out[t,:] = sum over s ascending with pair_row[t,s] >= 0 of topk_w[t,s] * y[pair_row[t,s],:]
 * (fp32 accumulation, one rounding to bf16).  A token with no local pair gives a zero row.
 *
 *   y_bf16    device, bf16 [n_rows,H], n_rows > max(pair_row)
 *   pair_row  device, int32 [T,k]
 *   topk_w    device, fp32 [T,k]
 *   out_bf16  device, bf16 [T,H] (out)
 *
 * Limits: H % 8 == 0, 1 <= k <= 8.  No workspace.
 */
int probe_combine(const void* y_bf16, const int32_t* pair_row, const float* topk_w, int T,
                  int H, int k, void* out_bf16, void* stream);

/* Combine for a model with a shared expert (one that every token uses, outside the gate; the paper's
 * Sec. 1 models include such, and the block's output is then the routed sum plus the shared expert's
 * output, Eq. 12 of the DeepSeek-V3 technical report without the residual connection):
 *   out[t,:] = sum_s topk_w[t,s] * y[pair_row[t,s],:]  +  shared_scale * shared_y[t,:]
 * added after the k routed terms, same fp32 accumulator, one rounding to bf16.
 *   shared_y_bf16  device, bf16 [T,H]: the shared expert's FFN output of every token, e.g. from
 *                  probe_grouped_ffn on x itself with one slot of T rows (slot_offsets = {0, T})
 * Other arguments and limits as probe_combine.
 */
int probe_combine_shared(const void* y_bf16, const int32_t* pair_row, const float* topk_w,
                         const void* shared_y_bf16, float shared_scale, int T, int H, int k,
                         void* out_bf16, void* stream);

/* Router of layer L-1 and predictor of layer L (residual at its zero initialisation) in one pass
 * over the same hidden states: the predictor reads the tensor that the previous layer's own gate
 * reads (Sec. 4.2), so the two gates can be stacked into one operand.  Results are those of
 * probe_route_topk(x, w_gate, bias, ...) and probe_predict_topk(x, w_gate_next, bias_next, ...) up to
 * fp32 summation order; x is read once and the split-K partial sums are half as many.
 * Both biases use the same bias_groups / tokens_per_group; either may be NULL.  pred_probs and probs
 * may be NULL.  Limits as probe_route_topk.
 */
size_t probe_route_predict_topk_workspace_bytes(int T, int H, int E, int k);

int probe_route_predict_topk(const void* x_bf16, const float* w_gate, const float* bias,
                             const float* w_gate_next, const float* bias_next, int bias_groups,
                             int tokens_per_group, int T, int H, int E, int k, int renormalize,
                             int32_t* topk_idx, float* topk_w, float* probs, int32_t* expert_counts,
                             int32_t* pred_idx, float* pred_w, float* pred_probs, int32_t* pred_counts,
                             void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------ packed gate ---
 *
 * The router's weights are frozen while serving (Sec. 4.2: the predictor clones (W_L, b_L)), so the
 * split of the fp32 gate into the three bf16 planes that the matrix cores consume can be done once
 * instead of inside every call.  probe_pack_gate writes them; the *_packed entry points take the planes
 * in place of the fp32 matrix and are otherwise the calls of the same name: same arithmetic, same
 * results bit for bit, a workspace smaller by the planes.
 *
 *   packed      device, bf16 [3][stack_rows][H], probe_pack_gate_bytes(H, stack_rows) bytes; plane p holds
 *               for every weight the round-to-nearest bf16 of what planes 0..p-1 left of it
 *   stack_rows  rows per plane; E for a single gate.  probe_route_predict_topk_packed takes one stack of
 *               2E rows: this layer's gate packed at row_offset 0, the next layer's at row_offset E
 *   row_offset  first row of this gate inside each plane
 * Limits: H % 8 == 0.  The planes are read-only afterwards and may be shared by any number of calls.
 */
size_t probe_pack_gate_bytes(int H, int stack_rows);

int probe_pack_gate(const float* w_gate, int H, int E, int stack_rows, int row_offset, void* packed,
                    void* stream);

size_t probe_route_topk_packed_workspace_bytes(int T, int H, int E, int k);

int probe_route_topk_packed(const void* x_bf16, const void* packed_gate, const float* bias,
                            int bias_groups, int tokens_per_group, int T, int H, int E, int k,
                            int renormalize, int32_t* topk_idx, float* topk_w, float* probs,
                            int32_t* expert_counts, void* workspace, size_t workspace_bytes,
                            void* stream);

/* workspace: probe_route_topk_packed_workspace_bytes */
int probe_predict_topk_packed(const void* h_prev_bf16, const void* packed_gate_next,
                              const float* bias_next, int bias_groups, int tokens_per_group, int T,
                              int H, int E, int k, int renormalize, int32_t* pred_idx, float* pred_w,
                              float* probs, int32_t* pred_counts, void* workspace,
                              size_t workspace_bytes, void* stream);

/* workspace: probe_route_topk_packed_workspace_bytes */
int probe_route_grouped_packed(const void* x_bf16, const void* packed_gate, const float* bias,
                               int bias_groups, int tokens_per_group, const float* select_bias,
                               const probe_gating* gating, int T, int H, int E, int k,
                               int32_t* topk_idx, float* topk_w, float* scores, int32_t* expert_counts,
                               void* workspace, size_t workspace_bytes, void* stream);

size_t probe_route_predict_topk_packed_workspace_bytes(int T, int H, int E, int k);

int probe_route_predict_topk_packed(const void* x_bf16, const void* packed_stack, const float* bias,
                                    const float* bias_next, int bias_groups, int tokens_per_group,
                                    int T, int H, int E, int k, int renormalize, int32_t* topk_idx,
                                    float* topk_w, float* probs, int32_t* expert_counts,
                                    int32_t* pred_idx, float* pred_w, float* pred_probs,
                                    int32_t* pred_counts, void* workspace, size_t workspace_bytes,
                                    void* stream);

/* ---------------------------------------------------------------------------- planner ---
 *
 * Greedy balance-optimal planning (Sec. 4.3, Algorithm 1) on the device: from the all-gathered
 * prediction to the plan probe_permute consumes, without a host round trip.
 *
 * Baseline placement P': expert e lives on rank e / E_loc.  The loop repeatedly takes the rank with
 * the largest latency L_r (bottleneck) and the valid rank with the smallest (helper), copies the
 * bottleneck's heaviest movable expert to the helper if both transfer budgets allow it, lets the
 * helper's own tokens of that expert stay at home (locality first) and redirects tokens whose origin
 * holds no copy from the bottleneck to the helper until the bottleneck's token load is down to the
 * cluster average (water-filling).  A move is kept when it lowers max_r L_r by more than eps; at most
 * k_max moves.  The paper names the terms of L_r but not their constants; here
 *     L_r = g_den * sum_{e: n_{e,r} > 0} (n_{e,r} + n0) + 2 * g_num * max(V_in_r, V_out_r)
 * (eta_g(n) = n / (n + n0) of Sec. 3.2; V_in / V_out = tokens received from / sent to other ranks,
 * Sec. 3.3, no deduplication).  All arithmetic is integer; ties go to the lower rank / expert id.
 */
typedef struct {
  int32_t max_replicas; /* replica slots per rank, |Delta^in_r| <= min(max_replicas, budget); <= 8 */
  int32_t budget;       /* experts a rank may send and may receive inside the hiding window; <= 8   */
  int32_t k_max;        /* accepted moves at most (Sec. 5 uses 16); <= 64                             */
  int64_t eps;          /* a move must lower the bottleneck latency by more than this                */
  int64_t n0;           /* tokens at which a grouped GEMM reaches half of its peak rate              */
  int64_t g_num, g_den; /* network time per token / compute time per token, g_den >= 1               */
} probe_planner_params;

/*
 *   n_hat        device, int32 [R,E]  tokens that originate on rank rs and are predicted for expert e
 *                (negative entries are read as 0)
 *   rank         the rank whose view of the plan is written to rep_off / rep_slot / rep_weight
 *   params       host pointer
 *   rep_off      device, int32 [E+1]                    (out)  } the probe_plan arrays: one replica per
 *   rep_slot     device, int32 [E + R*max_replicas]     (out)  } rank that holds the expert, ascending
 *   rep_weight   device, int32 [E + R*max_replicas]     (out)  } rank; weight = tokens planned for it
 *                (an expert with no predicted token keeps weight 1 on its home copy); local slots:
 *                native experts 0..E_loc-1, then replicas in the order they were added
 *   slot_expert  device, int32 [E_loc + max_replicas]   (out)  expert each local slot must hold, -1 = none
 *   delta_in     device, int32 [R,max_replicas]         (out)  experts copied onto each rank, -1 padded
 *   delta_out    device, int32 [R,budget] or NULL       (out)  experts each rank sends, -1 padded
 *   moves        device, int32 [k_max,3]                (out)  (expert, r_src, r_dst) per accepted move
 *   stats        device, int64 [4]  (out)  max L before, max L after, max token load after, moves
 *   n_assign     device, int32 [R,E,R] or NULL          (out)  tokens by (origin, expert, processing rank)
 * Limits: R <= 16, E <= 256, E_loc * R >= E.  One workgroup; meant to run beside the main track.
 */
size_t probe_plan_greedy_workspace_bytes(int R, int E);

int probe_plan_greedy(const int32_t* n_hat, int R, int E, int E_loc, int rank,
                      const probe_planner_params* params, int32_t* rep_off, int32_t* rep_slot,
                      int32_t* rep_weight, int32_t* slot_expert, int32_t* delta_in, int32_t* delta_out,
                      int32_t* moves, int64_t* stats, int32_t* n_assign, void* workspace,
                      size_t workspace_bytes, void* stream);

/* The plan of probe_plan_greedy as the SOURCE rank applies it to its own tokens ahead of the dispatch
 * exchange (assignment A of Sec. 3.1; locality first, Sec. 4.3), in the layout of probe_plan.  A slot
 * here is one (destination rank, expert copy) pair, numbered by destination rank first and expert
 * second; expert e lists its copies by ascending rank, rep_slot = the copy's slot, rep_weight =
 * n_assign[rank][e][r], the tokens from this origin planned for the copy on r.  With no token of e
 * predicted from this origin, an unforeseen one stays here if this rank holds a copy and goes to e's
 * home otherwise (weight 1).  probe_permute with this plan (num_slots = E + R*max_replicas) groups this
 * rank's pairs by destination rank and, inside a rank, by expert: slot_offsets[rank_off[r]] ..
 * slot_offsets[rank_off[r+1]] are the rows of xp to send to rank r.
 *   n_assign, delta_in  device, as written by probe_plan_greedy
 *   rep_off      device, int32 [E+1]                    (out)
 *   rep_slot     device, int32 [E + R*max_replicas]     (out)
 *   rep_weight   device, int32 [E + R*max_replicas]     (out)
 *   rank_off     device, int32 [R+1]                    (out) first slot of every destination rank
 *   slot_expert  device, int32 [E + R*max_replicas]     (out) expert of each slot in use
 * Limits as probe_plan_greedy.  No workspace.
 */
int probe_plan_dispatch(const int32_t* n_assign, const int32_t* delta_in, int R, int E, int E_loc,
                        int max_replicas, int rank, int32_t* rep_off, int32_t* rep_slot,
                        int32_t* rep_weight, int32_t* rank_off, int32_t* slot_expert, void* stream);

/* ---------------------------------------------------------------------------- metrics ---
 *
 * Evaluation of the lookahead predictor against the router it forecasts (Sec. 4.2, Sec. 6.4); not
 * on the serving path.
 *   hits = sum_t |{pred_idx[t,0..kp)} intersect {true_idx[t,0..kt)}|   (int64, exact)
 *       kp = kt = k: hits / (T k) is the top-k accuracy; kt = k/2: hits / (T k/2) is the top-half-k
 *       hit rate (true_idx lists a token's experts by descending logit)
 *   cross_entropy_sum = sum_t - sum_e true_probs[t,e] log pred_probs[t,e]  (fp64, fixed order),
 *       the loss of the online distillation; NULL to skip (then the probability tensors are not read)
 *   pred_idx / true_idx  device, int32, row t at t * stride;  pred_probs / true_probs  device, fp32 [T,E]
 *   hits  device int64 [1],  cross_entropy_sum  device double [1] or NULL
 */
int probe_predictor_metrics(const int32_t* pred_idx, int pred_stride, int kp, const int32_t* true_idx,
                            int true_stride, int kt, int T, const float* pred_probs,
                            const float* true_probs, int E, int64_t* hits, double* cross_entropy_sum,
                            void* stream);

#ifdef __cplusplus
}
#endif
#endif /* PROBE_H_ */
