/*
 * tamoe.h - C ABI of the one-device hot path of TA-MoE
 * ("TA-MoE: Topology-Aware Large Scale Mixture-of-Expert Training", NeurIPS 2022)
 * for AMD MI355X (gfx950).
 *
 * The path, for one device (rank) i of an expert-parallel MoE layer, in the paper's
 * notation (Section 3.1): N experts, P devices, E = N/P experts per device (device j holds
 * experts jE .. (j+1)E-1), S tokens on this device, k experts selected per token, hidden
 * size d:
 *
 *   tamoe_topo_pattern  host, once per topology: target dispatch pattern, penalty, capacity
 *   tamoe_gate          scores x W^T, softmax, top-k, load statistics
 *   tamoe_aux_loss      topology-aware auxiliary loss l_topo (or the plain l_aux)
 *   tamoe_dispatch      capacity-limited slot assignment + scatter into the send buffer
 *   tamoe_gate_dispatch the three calls above in one (three launches instead of seven)
 *   tamoe_combine       weighted gather of the returned rows into y
 * and around them
 *   tamoe_gate_bwd, tamoe_combine_bwd, tamoe_dispatch_bwd   backward of the path
 *   tamoe_regroup       received rows regrouped per local expert (and back)
 *   tamoe_penalty, tamoe_renorm_topk(_bwd), tamoe_dispatch_padded   variants: Norm of the penalty,
 *                       renormalised weights, fixed-size zero-padded send layout
 *   tamoe_tree_levels, tamoe_ring_table, tamoe_minmax_pattern   host: topology front-end
 *   tamoe_trace_*       kernel timing aid (HIP events around the launches), not a step of the path
 *
 * The global exchange, the experts and the return exchange sit between tamoe_dispatch and
 * tamoe_combine and are not part of this library.
 *
 * Conventions
 *  - Every matrix is row-major and dense.  Counts, indices and slots are int32_t.
 *  - "device" pointers are HIP device memory of the current device; "host" pointers are
 *    ordinary host memory.  The caller owns every buffer; the path's functions allocate nothing and
 *    keep no state between calls (two exceptions, both stated where they are declared: the built-in
 *    scratch of tamoe_dispatch_static and the process-wide kernel trace, which is off unless
 *    started).  Scratch comes from the caller's workspace `ws` (device
 *    memory, 256-byte aligned, at least tamoe_workspace_bytes() bytes).  Its content is
 *    garbage on entry and on exit; two calls that share a workspace must be ordered on one
 *    stream.
 *  - Device functions only enqueue work on `stream` (a hipStream_t passed as void*; NULL is
 *    the default stream).  They never synchronise and are deterministic: same inputs, same
 *    bits.
 *  - dtype: TAMOE_F32 (float), TAMOE_BF16 (bfloat16) or TAMOE_F16 (IEEE half precision, the FP16 of
 *    the paper's GPT model table); the 2-byte types are passed as bit patterns.
 *    A token row must be a multiple of 16 bytes (d % 4 == 0 for F32, d % 8 == 0 otherwise) and
 *    x, W, send, recv, y must be 16-byte aligned.
 *  - Limits: 1 <= N <= TAMOE_MAX_EXPERTS, 1 <= k <= min(N, TAMOE_MAX_K), N % P == 0,
 *    S * k < 2^31.  S = 0 is accepted by every device function except tamoe_aux_loss.
 *  - Inputs must be finite.  NaN scores give unspecified (but in-range or -1) selections.
 *  - Every function returns a tamoe_status.  On failure nothing has been enqueued and
 *    tamoe_last_error() describes the reason (thread-local, valid until the next call).
 */
#ifndef TAMOE_H
#define TAMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TAMOE_VERSION 1

#define TAMOE_MAX_EXPERTS 128
#define TAMOE_MAX_K 8

typedef enum tamoe_status {
    TAMOE_OK = 0,
    TAMOE_INVALID_ARG = 1,        /* null pointer, non-positive size, k > N, N % P != 0, rank
                                     outside [0,P), misaligned pointer, bad beta, bad level */
    TAMOE_UNSUPPORTED = 2,        /* dtype, N or k beyond the limits, row not a multiple of 16 B */
    TAMOE_WORKSPACE_TOO_SMALL = 3,
    TAMOE_HIP_ERROR = 4           /* a kernel launch was rejected by the HIP runtime */
} tamoe_status;

enum { TAMOE_F32 = 0, TAMOE_BF16 = 1, TAMOE_F16 = 2 };
enum { TAMOE_CAP_UNIFORM = 0, TAMOE_CAP_PROPORTIONAL = 1 };
enum { TAMOE_NORM_L1 = 0, TAMOE_NORM_SOFTMAX = 1 };

int tamoe_version(void);

/* Message of the last failure on the calling thread ("" if none). */
const char* tamoe_last_error(void);

/*
 * Setup, host only (all pointers host).  Section 4.2 "Model Optimization" and Section 4.3
 * "Routing Strategy" of the paper:
 *   1. if `level` is not NULL, smooth the profiled table per tree level: beta_l is the mean of
 *      beta[i][j] over the pairs i < j with level[i][j] == l (a label that occurs only on the
 *      diagonal takes the mean of those diagonal entries), beta_hat[i][j] = beta_{level[i][j]}
 *      (the hierarchical matrix); with level == NULL, beta is used as it is;
 *   2. target pattern of device `rank` (closed-form solution of the min-max exchange problem,
 *      latency dropped):
 *        c_hat[e] = k*S / ( E * (sum_{j=0..P-1} 1/beta_hat[rank][j]) * beta_hat[rank][e/E] );
 *   3. penalty[e] = (1/c_hat[e]) / sum_e' (1/c_hat[e'])          (p_i = Norm(1/c_hat_i));
 *   4. cap[e] = ceil(capacity_factor * k*S/N)      for cap_mode TAMOE_CAP_UNIFORM,
 *               ceil(capacity_factor * c_hat[e])   for cap_mode TAMOE_CAP_PROPORTIONAL
 *      (local capacity C_ie, Section 3.1 / Section 4.3; a product within 1e-9 of an integer
 *      counts as that integer).
 * beta  [P*P] inverse bandwidth of every device pair, diagonal included, all > 0 and finite.
 * level [P*P] non-negative tree-level label of every pair, or NULL.
 * Outputs (each may be NULL to skip it): c_hat [N] double, penalty [N] float, cap [N] int32.
 */
int tamoe_topo_pattern(const double* beta, const int32_t* level, int P, int N, int rank, int k,
                       int64_t S, double capacity_factor, int cap_mode,
                       double* c_hat, float* penalty, int32_t* cap);

/*
 * Penalty from a target pattern with a chosen Norm, host only (Section 4.3: p_i = Norm(1/c_hat_i);
 * besides the plain normalisation, functions that enlarge the penalty of slow transfers, softmax
 * for one, are admissible).
 *   TAMOE_NORM_L1:       penalty[e] = (1/c_hat[e]) / sum_e' (1/c_hat[e'])   (what tamoe_topo_pattern returns)
 *   TAMOE_NORM_SOFTMAX:  r[e] = (1/c_hat[e]) / mean_e' (1/c_hat[e']),
 *                        penalty[e] = exp(temperature * r[e]) / sum_e' exp(temperature * r[e'])
 * The paper leaves the scale of the softmax argument open; it is the explicit `temperature` here
 * (>= 0; 0 gives 1/N; ignored for TAMOE_NORM_L1).  On a two-tier pattern with bandwidth ratio rho
 * the slow/fast penalty ratio exceeds the L1 ratio rho once temperature > ln(rho) / (r_slow - r_fast).
 * c_hat [N] double (> 0, finite), penalty [N] float: host.
 */
int tamoe_penalty(const double* c_hat, int N, int norm, double temperature, float* penalty);

/*
 * Topology front-end, host only: tables for tamoe_topo_pattern from a description of the network
 * (Section 3.2: ring, symmetric and asymmetric tree in nested-list notation; Section 4.2).
 *
 * tamoe_tree_levels: `tree` is the paper's nested list as text: an integer n is a switch with n
 * devices, a list "[a,b,...]" a switch that joins its elements ("[2,2]": 2 switches x 2 devices;
 * "[[2,2],[2]]": the asymmetric 3-layer example).  Devices are numbered left to right.
 * level[i*P+j] = height of the lowest switch that joins devices i and j (1 = same device switch),
 * 0 on the diagonal: the labels tamoe_topo_pattern smooths over.  merge_asymmetric != 0 first merges
 * the tree (Section 4.2, last paragraph: separate nodes join the close symmetric sub-trees so that the
 * tree becomes symmetric; "[[2,2],[2]]" becomes "[[2,2,2]]").  The paper shows that one example; the
 * rule is this library's reading: one pass from the leaves up; at a list whose elements are all lists,
 * the elements with the most members are the full sub-trees, the smaller ones the separate nodes; each
 * separate node, left to right, hands all its members to one full sub-tree of its own height: the
 * one that has received the fewest members so far, the nearest of those, the left one at equal
 * distance.  Sizes are taken once, before anything moves.  The result is symmetric when the separate
 * nodes can be shared out equally ("[[2,2],[2,2],[2],[2]]" -> "[[2,2,2],[2,2,2]]"); otherwise it stays
 * asymmetric with its layers kept ("[[2,2],[2,2],[2]]" -> "[[2,2],[2,2,2]]").  Device switches are
 * never merged ("[3,1,2]" stays).  Devices keep the numbers of the tree as given, wherever the merge
 * moves their switch.
 * level: room for max_P*max_P ints; *P_out = devices found; tree_out (may be NULL): the tree that
 * was labelled, as text; device_order (may be NULL, room for max_P ints): the device numbers in the
 * order in which that tree lists them (0..P-1 unless the merge moved a switch past others).
 *
 * tamoe_ring_table: link q joins devices q and (q+1) mod P (inverse bandwidth beta_link[q] > 0,
 * latency alpha_link[q] >= 0 or alpha_link == NULL).  Other pairs hop over the devices between
 * them and the slowest link of the way dominates (Section 3.2): of the two arcs the one with the
 * smaller largest beta is used, on a tie the shorter, then the ascending one.  beta[i][j] = that
 * largest beta, alpha[i][j] (alpha may be NULL) = sum of the arc's latencies, level[i][j] = hops;
 * the diagonal gets self_beta, self_alpha, level 0.  All tables [P*P].
 *
 * tamoe_minmax_pattern: the exchange problem of Section 4.1 / 4.2 for one sender with the latency
 * term kept:  minimise over v >= 0, sum_j v_j = k*S:  max_j ( alpha_row[j] + beta_row[j] *
 * bytes_per_row * v_j ),  solved exactly; c_hat[e] = v_{e/E} / E, *t_comm (may be NULL) = the
 * optimum.  With alpha_row == NULL or constant it returns the closed form that
 * tamoe_topo_pattern uses.  The balance constraint across senders is not imposed (as in the
 * closed form, where it holds by symmetry of the table).
 */
int tamoe_tree_levels(const char* tree, int merge_asymmetric, int max_P, int32_t* level, int* P_out,
                      char* tree_out, size_t tree_out_len, int32_t* device_order);
int tamoe_ring_table(const double* beta_link, const double* alpha_link, int P, double self_beta,
                     double self_alpha, double* beta, double* alpha, int32_t* level);
int tamoe_minmax_pattern(const double* alpha_row, const double* beta_row, int P, int N, int k, int64_t S,
                         double bytes_per_row, double* c_hat, double* t_comm);

/* Bytes of device workspace that any of the device functions below needs for this shape and storage
 * type (fp32 storage adds room for the partial scores of the gate's K split).  Grows with S. */
size_t tamoe_workspace_bytes(int64_t S, int d, int N, int P, int k, int dtype);

/*
 * Gate (Section 3.1: gate network G, softmax, top-k; load statistics of Section 3.1 / 4.1).
 *   logits[t][e]  = sum_q x[t][q] * W[e][q]             (fp32 accumulation)
 *   G[t][:]       = softmax over the N experts of logits[t][:]
 *   topk_idx[t][j], j = 0..k-1: the k experts with the highest logits, best first, equal
 *                   logits to the lower expert index;  topk_w[t][j] = G[t][topk_idx[t][j]]
 *                   (not renormalised over the k choices)
 *   c_expert[e]   = number of (t, j) with topk_idx[t][j] == e        (before any capacity)
 *   c_device[j]   = sum of c_expert over the experts of device j
 *   m[e]          = (1/S) * sum_t G[t][e]                             (0 if S == 0)
 * x [S,d], w [N,d]: device, `dtype`.   logits [S,N] float, device, may be NULL.
 * topk_idx [S,k] int32, topk_w [S,k] float, m [N] float, c_expert [N] int32,
 * c_device [P] int32: device outputs.  The selection is taken on exactly the fp32 logits that
 * are written to `logits`.
 */
int tamoe_gate(const void* x, const void* w, int dtype, int64_t S, int d, int N, int P, int k,
               float* logits, int32_t* topk_idx, float* topk_w, float* m,
               int32_t* c_expert, int32_t* c_device,
               void* ws, size_t ws_bytes, void* stream);

/*
 * The gate's selection stage on given scores: everything tamoe_gate computes after the matrix
 * product, from logits [S,N] float (device).  Same outputs, same arithmetic.
 */
int tamoe_select(const float* logits, int64_t S, int N, int P, int k,
                 int32_t* topk_idx, float* topk_w, float* m,
                 int32_t* c_expert, int32_t* c_device,
                 void* ws, size_t ws_bytes, void* stream);

/*
 * Auxiliary loss (Section 4.3, the topology loss; Section 3.1, the load-balance loss).
 *   penalty != NULL:  loss = N*P * sum_e penalty[e] * m[e] * c_expert[e] / S      (l_topo)
 *   penalty == NULL:  loss =       sum_e              m[e] * c_expert[e] / S      (l_aux)
 * m [N] float, c_expert [N] int32, penalty [N] float, loss [1] float: device.  S > 0.
 */
int tamoe_aux_loss(const float* m, const int32_t* c_expert, const float* penalty,
                   int N, int P, int64_t S, float* loss, void* stream);

/*
 * Capacity-limited dispatch (Section 3.1: dispatched data [k*S, d], [c_ie, d] per expert, local
 * capacity c_ie <= C_ie; Section 4.1: chunks for one device merged into one delivery; Section
 * 4.3: variable chunk sizes instead of zero padding).
 * Pairs (t, j) are ranked choice-major: all first choices in token order, then all second
 * choices, ...  pos(t,j) = number of earlier pairs with the same expert e = topk_idx[t][j].
 * The pair is kept iff pos < cap[e].
 *   kept_expert[e]    = min(c_expert[e], cap[e])
 *   expert_offset[e]  = sum_{e' < e} kept_expert[e'],  expert_offset[N] = K (rows in `send`)
 *   slot[t][j]        = expert_offset[e] + pos  if kept, else -1
 *   send_count_dev[j] = sum of kept_expert over the experts of device j  (rows bound for j)
 *   send[slot[t][j]][:] = x[t][:]   bit copy, for every kept pair
 * so `send` lists rows expert by expert, hence destination device by destination device.
 * An index outside [0, N) in topk_idx is treated as a dropped pair (slot -1, not counted).
 * x [S,d] `dtype`, topk_idx [S,k], cap [N] (>= 0): device inputs.  send: device, room for k*S
 * rows of d elements; only the first K rows are written.  slot [S,k], kept_expert [N],
 * expert_offset [N+1], send_count_dev [P]: device outputs.
 */
int tamoe_dispatch(const void* x, const int32_t* topk_idx, const int32_t* cap, int dtype,
                   int64_t S, int d, int N, int P, int k,
                   void* send, int32_t* slot, int32_t* kept_expert, int32_t* expert_offset,
                   int32_t* send_count_dev,
                   void* ws, size_t ws_bytes, void* stream);

/*
 * The forward path up to the send buffer in one call and three kernel launches: tamoe_gate,
 * tamoe_aux_loss and tamoe_dispatch fused (Section 3.1: gate, softmax, top-k, load statistics, local
 * capacity; Section 4.1: per-device delivery; Section 4.3: l_topo, variable chunk sizes).  Layers of the
 * paper's own size (hidden size 1024, a few thousand tokens per device) are bound by the number of
 * launches, not by bytes; the gate kernel hands the slot assignment what it needs (pairs per gate
 * workgroup, expert and choice; every pair's position inside its workgroup), so that no kernel has
 * to read the routing again.
 * Every output is defined as in the three separate calls, with the gate's own topk_idx as the routing:
 *   logits (may be NULL), topk_idx, topk_w, m, c_expert, c_device     as tamoe_gate
 *   loss (may be NULL)      l_topo with `penalty`, l_aux with penalty == NULL   as tamoe_aux_loss (0 if S == 0)
 *   send, slot, kept_expert, expert_offset, send_count_dev            as tamoe_dispatch with `cap`
 * Integer outputs and the send buffer are bit-identical to the separate calls'; topk_w is bit-identical;
 * m and loss may differ from theirs in the last bits (another fixed summation order).
 * penalty [N] float or NULL, cap [N] int32: device.  ws: tamoe_workspace_bytes(S, d, N, P, k, dtype).
 */
int tamoe_gate_dispatch(const void* x, const void* w, int dtype, int64_t S, int d, int N, int P, int k,
                        const float* penalty, const int32_t* cap,
                        float* logits, int32_t* topk_idx, float* topk_w, float* m,
                        int32_t* c_expert, int32_t* c_device, float* loss,
                        void* send, int32_t* slot, int32_t* kept_expert, int32_t* expert_offset,
                        int32_t* send_count_dev,
                        void* ws, size_t ws_bytes, void* stream);

/*
 * tamoe_dispatch for callers that cannot allocate device memory or carry a workspace (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): same arguments, outputs and
 * kernels as tamoe_dispatch without `ws`.  The pair counters live in an array inside the library's
 * own device image, TAMOE_STATIC_SCRATCH_BYTES per device, held until the process ends; the call
 * allocates and frees nothing.  Limit: k * ceil(S/1024) * N * 4 <= TAMOE_STATIC_SCRATCH_BYTES
 * (k = 2, N = 128: S <= 1 048 576), else TAMOE_UNSUPPORTED.  Every call on a device uses that
 * device's one array: calls that overlap on one device (two streams, two threads) race; order them.
 * The array's content between calls is garbage (every counter is written before it is read).
 * The first call on a device looks up the array's address, so make that call outside a capture.
 */
#define TAMOE_STATIC_SCRATCH_BYTES (1 << 20)
int tamoe_dispatch_static(const void* x, const int32_t* topk_idx, const int32_t* cap, int dtype,
                          int64_t S, int d, int N, int P, int k,
                          void* send, int32_t* slot, int32_t* kept_expert, int32_t* expert_offset,
                          int32_t* send_count_dev, void* stream);

/*
 * Weighted combine (Section 3.1: the output y of the layer aggregates the computed results).
 * recv holds the expert outputs in the row order of the send buffer.
 *   y[t][:] = sum over j = 0..k-1 with slot[t][j] >= 0 of topk_w[t][j] * recv[slot[t][j]][:]
 * accumulated in fp32 in ascending j and rounded once to `dtype`; a token whose choices were
 * all dropped gets a zero row.  A slot >= K_rows is ignored like a dropped pair.
 * recv [K_rows,d] `dtype`, slot [S,k], topk_w [S,k] float: device inputs; y [S,d]: device out.
 */
int tamoe_combine(const void* recv, int64_t K_rows, const int32_t* slot, const float* topk_w,
                  int dtype, int64_t S, int d, int k, void* y, void* stream);

/*
 * Backward of the path (training adds the auxiliary loss to the train loss, Sections 3.1 and 4.3,
 * so its gradient and the transposes of the two row movers are needed).  Routing is fixed: the
 * selected indices, the counts and the slots are constants of the differentiation.
 *
 * tamoe_gate_bwd: gradient to the gate scores.  With L = sum_{t,j} d_topk_w[t][j] * G[t][idx[t][j]]
 * + loss_scale * l_topo (penalty != NULL; l_aux if penalty == NULL) and the softmax Jacobian,
 *   u[t][e]        = sum_j d_topk_w[t][j] * [topk_idx[t][j] == e] + loss_scale * N*P * penalty[e] * c_expert[e] / S^2
 *   d_logits[t][e] = G[t][e] * ( u[t][e] - sum_e' u[t][e'] * G[t][e'] ),     G = softmax(logits[t][:])
 * (for l_aux: the factor N*P*penalty[e] is 1).  logits [S,N] float, topk_idx [S,k], d_topk_w [S,k]
 * float, penalty [N] float or NULL, c_expert [N]: device inputs; d_logits [S,N] float: device out.
 */
int tamoe_gate_bwd(const float* logits, const int32_t* topk_idx, const float* d_topk_w,
                   const float* penalty, const int32_t* c_expert, float loss_scale,
                   int64_t S, int N, int P, int k, float* d_logits, void* stream);

/*
 * tamoe_combine_bwd: transpose of tamoe_combine for an upstream gradient dy [S,d] (`dtype`):
 *   d_recv[slot[t][j]][:] = topk_w[t][j] * dy[t][:]              rounded once to `dtype`, kept pairs
 *   d_topk_w[t][j]        = sum_q dy[t][q] * recv[slot[t][j]][q] fp32, 0 for a dropped pair
 * Every row of the send buffer is named by exactly one kept pair, so rows 0..K-1 of d_recv are
 * all written; rows that no slot names are left untouched.  dy [S,d], recv [K_rows,d], slot [S,k],
 * topk_w [S,k]: device inputs; d_recv [K_rows,d] `dtype`, d_topk_w [S,k] float: device outputs.
 */
int tamoe_combine_bwd(const void* dy, const void* recv, int64_t K_rows, const int32_t* slot,
                      const float* topk_w, int dtype, int64_t S, int d, int k,
                      void* d_recv, float* d_topk_w, void* stream);

/*
 * tamoe_dispatch_bwd: transpose of the scatter of tamoe_dispatch for the gradient d_send [K_rows,d]
 * that arrives at the send buffer:  d_x[t][:] = sum over kept j of d_send[slot[t][j]][:], fp32
 * accumulation, one rounding to `dtype`; zero row for a token with no kept choice.
 */
int tamoe_dispatch_bwd(const void* d_send, int64_t K_rows, const int32_t* slot, int dtype,
                       int64_t S, int d, int k, void* d_x, void* stream);

/*
 * Combine weights renormalised over the k selected experts of a token (a variant of the weighting
 * G(x)_e of Section 3.1 in which a token's k weights sum to one; taken before any capacity drop):
 *   out[t][j] = topk_w[t][j] / (topk_w[t][0] + ... + topk_w[t][k-1])      fp32, sum in ascending j
 * and its transpose for a gradient d_out [S,k] that arrives at the renormalised weights:
 *   d_topk_w[t][i] = d_out[t][i] / s - (sum_j d_out[t][j] * topk_w[t][j]) / s^2,   s = sum_j topk_w[t][j]
 * (feed d_topk_w to tamoe_gate_bwd).  All pointers device, [S,k] float; out may alias topk_w and
 * d_topk_w may alias d_out.
 */
int tamoe_renorm_topk(const float* topk_w, int64_t S, int k, float* out, void* stream);
int tamoe_renorm_topk_bwd(const float* topk_w, const float* d_out, int64_t S, int k, float* d_topk_w,
                          void* stream);

/*
 * Dispatch into the fixed-size zero-padded layout that the variable chunk sizes of Section 4.3
 * replace: every expert owns C rows of `send` whether it fills them or not (so every destination
 * device receives E*C rows).  Same pair order as tamoe_dispatch; a pair is kept iff
 * pos < min(cap[e], C) (cap == NULL: pos < C).
 *   kept_expert[e]  = min(c_expert[e], cap[e], C)
 *   slot[t][j]      = e*C + pos  if kept, else -1
 *   send[slot[t][j]][:] = x[t][:];  rows e*C + kept_expert[e] .. (e+1)*C - 1 are set to zero
 * tamoe_combine works on this layout unchanged (K_rows = N*C).
 * send: device, [N*C, d] `dtype`, every row written; N*C < 2^31.  Other arguments as tamoe_dispatch.
 */
int tamoe_dispatch_padded(const void* x, const int32_t* topk_idx, const int32_t* cap, int dtype,
                          int64_t S, int d, int N, int P, int k, int C,
                          void* send, int32_t* slot, int32_t* kept_expert,
                          void* ws, size_t ws_bytes, void* stream);

/*
 * Receive side: regroup the rows of the global exchange per local expert (Section 3.1: each
 * expert receives a combined batch of tokens; rows from process s for expert e: c_se).
 * The receive buffer `in` holds one chunk per source device s = 0..P-1, in that order; inside a
 * chunk the rows are grouped by local expert e = 0..E-1, recv_count[s*E + e] rows each
 * (source-major).  Expert-major lists, for e = 0..E-1, the segments of s = 0..P-1 in that order,
 * so that every local expert has one contiguous batch.
 *   to_expert_major != 0: in is source-major, out becomes expert-major (before the experts);
 *   to_expert_major == 0: the inverse (before the return exchange).
 * expert_offset [E+1] (may be NULL): first row of every expert's batch, expert_offset[E] = rows.
 * cap_rows = number of rows both buffers can hold; only the first R = sum of the counts rows are
 * read and written (R is taken on the device; rows beyond cap_rows are dropped).  P*E <= 128.
 * in, out [cap_rows, d] `dtype`, recv_count [P*E], expert_offset: device.  ws: at least
 * tamoe_workspace_bytes(...) (any shape) bytes.
 */
int tamoe_regroup(const void* in, const int32_t* recv_count, int P, int E, int dtype, int d,
                  int64_t cap_rows, int to_expert_major, void* out, int32_t* expert_offset,
                  void* ws, size_t ws_bytes, void* stream);

/*
 * Kernel timing aid for benchmarks (not a step of the path; off unless started).
 * tamoe_trace_start creates 2*max_launches HIP events on the current device; from then on every
 * kernel the device functions above enqueue is bracketed by a pair of events on its stream,
 * until max_launches kernels have been recorded or tamoe_trace_stop is called.
 * tamoe_trace_stop waits for the recorded events and returns the number of records (>= 0), or
 * a negative tamoe_status.  tamoe_trace_get copies record i: the kernel's name (truncated to
 * name_len-1 characters) and its duration in milliseconds.  tamoe_trace_clear destroys the
 * events.  tamoe_trace_filter restricts the bracketing to launches of the kernel with the given
 * name (NULL: every kernel again), so that a benchmark can time one kernel with two event records
 * per step instead of two per launch; it may be called at any time.
 * One trace at a time, process-wide: the records are shared by every thread that launches while it
 * runs (a lock serialises their bookkeeping; records of concurrent threads interleave).  Start, stop,
 * get and clear belong to one controlling thread.  All pointers host.
 */
int tamoe_trace_start(int max_launches);
int tamoe_trace_filter(const char* kernel_name);
int tamoe_trace_stop(void);
int tamoe_trace_get(int i, char* name, size_t name_len, float* ms);
int tamoe_trace_clear(void);

#ifdef __cplusplus
}
#endif
#endif /* TAMOE_H */
