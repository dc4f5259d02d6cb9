/*
 * moe_hip.h -- C ABI of the one-GPU MoE-layer hot path (MI355X / gfx950).
 *
 * The library computes one GPU's share of an MoE layer's training step, i.e. the
 * MoE layer of Eq. 3 of the paper
 *     MoE(x) = sum_{i in argtopk(g(x))} g(x)_i * f(x W_i^A) W_i^B
 * with the expert body of Eq. 1 (FFN(x) = f(x W^A) W^B) read as SwiGLU
 * (W^A = (Wg, Wu), f(x W^A) = silu(x Wg) * (x Wu), W^B = Wd), without token
 * dropping (evaluation setup of the paper: every assignment is computed), for
 * tokens whose experts are all local (the local branch of the paper's token
 * dispatching, Algorithm 3), and its backward pass.
 *
 * Conventions common to every entry point
 *  - Every pointer is a DEVICE pointer owned by the caller unless it says "host".
 *    The library never allocates, frees or keeps a pointer past the call.
 *  - All tensors are dense row-major; base pointers must be 16-byte aligned.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  A call
 *    only enqueues kernels on that stream and returns without synchronising.
 *  - dtype MOE_F32: X, weights, activations, outputs and weight gradients are fp32.
 *    dtype MOE_BF16: they are bfloat16 (round-to-nearest-even at every store),
 *    products accumulate in fp32.  Logits, combine weights and their gradient are
 *    always fp32; all index arrays are int32.
 *  - Return value: MOE_OK, or a negative error code; on error nothing was launched
 *    and moe_last_error() describes the reason (thread-local, host string).
 *  - Calls on one stream are ordered; two calls that share a workspace must not
 *    overlap.
 *  - Empty inputs are valid: with T == 0 (n_rows == 0 for the expert calls) a call succeeds,
 *    tensors with no elements may be null, and only the outputs that do not depend on tokens
 *    are written (counts and offsets = 0; n_active = 0, active_ids = -1).
 */
#ifndef MOE_HIP_H
#define MOE_HIP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MOE_ABI_VERSION 1

enum { MOE_F32 = 0, MOE_BF16 = 1 };
enum { MOE_GATE_SOFTMAX = 0, MOE_GATE_SIGMOID = 1 };
enum {
  MOE_OK = 0,
  MOE_EINVAL = -1,  /* null pointer, bad shape, bad alignment */
  MOE_EWS = -2,     /* workspace too small */
  MOE_EDTYPE = -3,  /* unknown dtype / gate */
  MOE_ELAUNCH = -4  /* the HIP runtime refused a launch */
};

/* Shape of the routed part of one MoE layer on this GPU. */
typedef struct moe_shape {
  int32_t T;      /* tokens on this GPU                                  (>= 0) */
  int32_t d;      /* hidden size; multiple of 8                                  */
  int32_t E;      /* routed experts, 1..MOE_MAX_EXPERTS                          */
  int32_t k;      /* experts per token, 1..min(E, MOE_MAX_TOPK)                  */
  int32_t d_ff;   /* expert width; multiple of 8                                 */
  int32_t dtype;  /* MOE_F32 or MOE_BF16                                         */
  int32_t gate;   /* MOE_GATE_SOFTMAX (over all E logits) or MOE_GATE_SIGMOID    */
  int32_t renorm; /* 1: the k selected scores are divided by their sum           */
} moe_shape_t;

#define MOE_MAX_EXPERTS 1024
#define MOE_MAX_TOPK 64

int moe_abi_version(void);
const char* moe_last_error(void);

/* Workspace sizes in bytes (host computation, no GPU call; 0 for invalid arguments).
 * n_groups/n_rows as passed to the expert calls, shared = 1 for shared mode (offsets == NULL);
 * `shape` supplies d, d_ff, dtype (and T, k, E for the dispatch). */
size_t moe_dispatch_workspace_bytes(const moe_shape_t* shape);
size_t moe_expert_fwd_workspace_bytes(const moe_shape_t* shape, int32_t n_groups, int32_t n_rows,
                                      int32_t shared);
size_t moe_expert_bwd_workspace_bytes(const moe_shape_t* shape, int32_t n_groups, int32_t n_rows,
                                      int32_t shared);

/*
 * moe_router_fwd / moe_router_bwd -- the gating network that produces the logits of Eq. 3, read
 * as one linear map without bias (the paper only calls it lightweight), and its adjoint:
 *   logits = X Wr;      dWr = X^T dlogits;   dX = dlogits Wr^T  (added to dX when accumulate != 0).
 *   X [T, d], Wr [d, E], dWr [d, E], dX [T, d] in shape->dtype; logits, dlogits [T, E] f32.
 * bf16 operands, fp32 accumulation; dlogits is rounded to bf16 for the two backward products.
 * E need not be a multiple of anything: the GEMMs run on zero-padded copies in the workspace
 * (moe_router_*_workspace_bytes, host computation).  With T == 0, moe_router_bwd writes dWr = 0.
 * These calls are not part of the path the benchmark times (logits are an input there).
 */
size_t moe_router_fwd_workspace_bytes(const moe_shape_t* shape);
size_t moe_router_bwd_workspace_bytes(const moe_shape_t* shape);
int moe_router_fwd(const moe_shape_t* shape, const void* X, const void* Wr, float* logits, void* ws, size_t ws_bytes,
                   void* stream);
int moe_router_bwd(const moe_shape_t* shape, const void* X, const void* Wr, const float* dlogits, void* dWr, void* dX,
                   int32_t accumulate, void* ws, size_t ws_bytes, void* stream);

/*
 * moe_route -- the gate of Eq. 3: g(x) and argtopk.
 *   logits   [T, E] f32  router logits
 *   topk_idx [T, k] i32  out: the k experts of each token, by descending logit; equal
 *                        logits go to the lower expert index (selection is on the raw
 *                        fp32 logits: softmax and sigmoid are increasing)
 *   topk_w   [T, k] f32  out: g(x)_i of the selected experts (softmax over all E, or
 *                        sigmoid), divided by their sum when shape->renorm
 * NaN logits are a caller error (result unspecified, no fault).
 */
int moe_route(const moe_shape_t* shape, const float* logits, int32_t* topk_idx, float* topk_w,
              void* stream);

/*
 * moe_route_bwd -- backward of the gate of Eq. 3 with the selection held fixed (top-k is
 * piecewise constant): the gradient of the loss with respect to the router logits from the
 * gradient dw of the combine weights (moe_combine_bwd).
 *   w_j = s_j / sum_i s_i (renorm) or s_j, s = softmax(logits) or sigmoid(logits):
 *   ds_j = (dw_j - sum_i dw_i w_i) / sum_i s_i (renorm) or dw_j;  ds_e = 0 for unselected e;
 *   softmax: dlogits_e = s_e (ds_e - sum_j s_j ds_j);   sigmoid: dlogits_e = ds_e s_e (1 - s_e).
 *   logits [T, E] f32;  topk_idx [T, k] i32 from moe_route;  dw [T, k] f32;
 *   dlogits [T, E] f32 out (every element is written)
 * topk_idx entries outside 0..E-1 are a caller error (result unspecified).
 */
int moe_route_bwd(const moe_shape_t* shape, const float* logits, const int32_t* topk_idx, const float* dw,
                  float* dlogits, void* stream);

/*
 * moe_aux_loss / moe_aux_loss_bwd -- the auxiliary load-balancing loss the paper's evaluation
 * setup trains with (Section 5.1, experimental setup: weight 0.001; its sensitivity study sweeps the
 * weight to 0.1).  The paper cites the loss and does not print it; this is the product form of that
 * family:
 *   L = alpha * E * sum_e f_e * P_e,   f_e = counts[e] / (T k),   P_e = (1/T) sum_t p_te,
 *   p_t = the gate's scores as shares of one: softmax(logits_t), or sigmoid(logits_t) divided by
 *   its sum over the E experts.  L = alpha when the loads or the scores are uniform.
 * The backward holds the loads f constant (they are piecewise constant in the logits):
 *   c_e = dloss alpha E f_e / T;  softmax: dlogits_te = p_te (c_e - sum_j p_tj c_j);
 *   sigmoid: dlogits_te = (c_e - sum_j p_tj c_j) / (sum_j s_tj) * s_te (1 - s_te).
 *   logits [T, E] f32 (device);  counts [E] i32 (device, from moe_dispatch);  alpha, dloss host scalars
 *   P [E] f32 out, loss [1] f32 out (device; both 0 when T == 0)
 *   ws >= moe_aux_loss_workspace_bytes(shape): per-wavefront partial sums, reduced in a fixed
 *   order (no atomics: two runs give identical bits)
 *   dlogits [T, E] f32: written, or added to when accumulate != 0 (e.g. after moe_route_bwd)
 * shape->renorm and shape->k's selection play no part beyond k in f_e.
 */
size_t moe_aux_loss_workspace_bytes(const moe_shape_t* shape);
int moe_aux_loss(const moe_shape_t* shape, const float* logits, const int32_t* counts, float alpha, float* P,
                 float* loss, void* ws, size_t ws_bytes, void* stream);
int moe_aux_loss_bwd(const moe_shape_t* shape, const float* logits, const int32_t* counts, float alpha,
                     float dloss, int32_t accumulate, float* dlogits, void* stream);

/*
 * moe_dispatch -- group the T*k token-expert assignments by expert and copy the token rows
 * into expert-contiguous order (the local-dispatch case of Algorithm 3: counts[e] is its
 * token assignment T[e, d] for this device; no token is dropped).
 *   X        [T, d]       tokens
 *   topk_idx [T, k]       from moe_route
 *   counts   [E]    i32   out: assignments per expert
 *   offsets  [E+1]  i32   out: exclusive prefix sum of counts, offsets[E] = T*k
 *   row_of   [T*k]  i32   out: row of assignment a = t*k + j in the grouped order; rows of
 *                         one expert are in ascending a (stable counting sort)
 *   src_of   [T*k]  i32   out: inverse of row_of
 *   Xp       [T*k, d]     out: Xp[row_of[a], :] = X[a / k, :]
 *   ws, ws_bytes          scratch of at least moe_dispatch_workspace_bytes(shape)
 * Entries of topk_idx outside [0, E) are a caller error; they are ignored (no fault) and the
 * outputs are then unspecified.
 */
int moe_dispatch(const moe_shape_t* shape, const void* X, const int32_t* topk_idx, int32_t* counts,
                 int32_t* offsets, int32_t* row_of, int32_t* src_of, void* Xp, void* ws,
                 size_t ws_bytes, void* stream);

/*
 * moe_route_dispatch -- moe_route, moe_dispatch and (with aux_P, aux_loss != NULL) moe_aux_loss in one call
 * of four kernels instead of seven: the gate of Eq. 3 and the counting of Algorithm 3's token assignment
 * read the logits once.  Same arguments and the same results as the three calls: every integer output
 * and topk_w bit for bit; aux_P and aux_loss up to the order of their fp32 sums (a fixed order, so two
 * runs agree bit for bit).  aux_alpha is ignored when aux_P and aux_loss are NULL (they go together).
 *   ws >= moe_route_dispatch_workspace_bytes(shape)
 * moe_route_aux_bwd -- moe_route_bwd followed by moe_aux_loss_bwd(accumulate = 1) in one kernel:
 *   dlogits = d(loss)/d(logits) through the combine weights (from dw) + dloss * d(aux loss)/d(logits).
 */
size_t moe_route_dispatch_workspace_bytes(const moe_shape_t* shape);
int moe_route_dispatch(const moe_shape_t* shape, const float* logits, const void* X, float aux_alpha,
                       int32_t* topk_idx, float* topk_w, int32_t* counts, int32_t* offsets, int32_t* row_of,
                       int32_t* src_of, void* Xp, float* aux_P, float* aux_loss, void* ws, size_t ws_bytes,
                       void* stream);
int moe_route_aux_bwd(const moe_shape_t* shape, const float* logits, const int32_t* topk_idx, const float* dw,
                      const int32_t* counts, float alpha, float dloss, float* dlogits, void* stream);

/*
 * moe_dispatch_static -- moe_dispatch for callers that cannot allocate device memory or cannot hand over
 * a workspace: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, same kernels and same results as moe_dispatch, without `ws`: the per-chunk
 * histograms live in an array that is part of the library's code object (4 * MOE_DISPATCH_STATIC_MAX_COUNTERS
 * bytes = 1 MiB on every GPU the library runs on, until the process ends).  The call allocates
 * nothing and frees nothing (with per-kernel timing off: moe_profile_enable creates events).
 *   limit: ceil(T*k / 256) * E <= MOE_DISPATCH_STATIC_MAX_COUNTERS, else MOE_EWS and nothing is launched
 *   (T*k = 65536 assignments over 1024 experts, or 2^20 assignments over 64 experts, fit).
 * Every call on one GPU uses that GPU's one array: two calls that overlap in time on the same GPU
 * (different streams) race; calls on one stream are ordered and need no clearing in between (every
 * counter a call reads was written by the same call).  The array's address is looked up once per
 * device on the first call with that device current; a failure there returns MOE_ELAUNCH.
 */
#define MOE_DISPATCH_STATIC_MAX_COUNTERS 262144
int moe_dispatch_static(const moe_shape_t* shape, const void* X, const int32_t* topk_idx, int32_t* counts,
                        int32_t* offsets, int32_t* row_of, int32_t* src_of, void* Xp, void* stream);

/*
 * moe_expert_fwd -- the expert bodies of Eq. 3 as a grouped GEMM over variable row counts.
 * Grouped mode (offsets != NULL): group e owns rows [offsets[e], offsets[e+1]) of Xin;
 *   G = Xin_e Wg[e], U = Xin_e Wu[e], H = silu(G) * U, Yout_e = H Wd[e].
 *   Groups without rows cost nothing (no tile, no weight read).
 * Shared mode (offsets == NULL): each of the n_groups always-on experts runs on ALL n_rows
 *   rows; G, U, H are [n_groups, n_rows, d_ff] and Yout is the sum over groups (Eq. 2).
 *   n_groups  experts (shape->E in grouped mode; shape->E is not otherwise used here)
 *   n_rows    rows of Xin (T*k in grouped mode, T in shared mode)
 *   Xin  [n_rows, d]; Wg, Wu [n_groups, d, d_ff]; Wd [n_groups, d_ff, d]
 *   G, U, H   out, [n_rows, d_ff] (shared: [n_groups, n_rows, d_ff]); kept for the backward pass
 *   Yout [n_rows, d]  out
 * shape->d_ff is the width of these experts (shared experts may use their own shape).
 * Two-matrix experts (Wu == NULL): Eq. 1 as the paper prints it, FFN(x) = f(x W^A) W^B with
 *   W^A = Wg, W^B = Wd and f = GELU, gelu(z) = z Phi(z) (the paper's synthetic GPT-MoE models;
 *   it does not name f): G = Xin_e Wg[e] (the pre-activation), H = gelu(G), Yout_e = H Wd[e];
 *   U is not touched and may be NULL.  In moe_expert_bwd the same mode (Wu == NULL) gives
 *   dG = (dYin Wd^T) * gelu'(G), gelu'(z) = Phi(z) + z phi(z); dXin = dG Wg^T; dWg = Xin^T dG;
 *   dWd = H^T dYin; U and dWu_c are not touched and may be NULL.
 */
int moe_expert_fwd(const moe_shape_t* shape, int32_t n_groups, const int32_t* offsets, int32_t n_rows,
                   const void* Xin, const void* Wg, const void* Wu, const void* Wd, void* G, void* U,
                   void* H, void* Yout, void* ws, size_t ws_bytes, void* stream);

/*
 * moe_expert_bwd -- backward of moe_expert_fwd (chain rule on Eq. 1):
 *   dH = dYin Wd^T;  s = sigmoid(G);  dU = dH * G * s;  dG = dH * U * s * (1 + G (1 - s));
 *   dXin = dG Wg^T + dU Wu^T;  dWg = Xin^T dG;  dWu = Xin^T dU;  dWd = H^T dYin  (per group).
 * The weight gradients are written COMPACTED to activated experts: active_ids lists, in
 * ascending order, the groups that own at least one row (n_active of them; the remaining
 * entries are -1) and slot i of dWg_c/dWu_c/dWd_c holds the gradient of group active_ids[i].
 * Slots >= n_active are not written.  This is the per-GPU list of gradient chunks that the
 * paper's SparseReduceScatter would send (one chunk per materialised expert, Eq. 4).
 * Shared mode (offsets == NULL): every group is active, dXin is the sum over groups.
 *   dYin [n_rows, d];  dXin [n_rows, d] out
 *   active_ids [n_groups] i32 out;  n_active [1] i32 out (device)
 *   dWg_c, dWu_c [n_groups, d, d_ff] out;  dWd_c [n_groups, d_ff, d] out
 *   ws >= moe_expert_bwd_workspace_bytes(shape, n_groups, n_rows, offsets == NULL)
 */
int moe_expert_bwd(const moe_shape_t* shape, int32_t n_groups, const int32_t* offsets, int32_t n_rows,
                   const void* Xin, const void* Wg, const void* Wu, const void* Wd, const void* G,
                   const void* U, const void* H, const void* dYin, void* dXin, int32_t* active_ids,
                   int32_t* n_active, void* dWg_c, void* dWu_c, void* dWd_c, void* ws,
                   size_t ws_bytes, void* stream);

/*
 * moe_expert_fwd_gather / moe_expert_bwd_gather -- the two expert calls in grouped mode (routed experts:
 * n_groups = shape->E, n_rows = shape->T * shape->k) reading token rows in place instead of permuted
 * copies: tokens whose experts are all local need no exchange (the local branch of Algorithm 3), so the
 * grouped order can be an index, src_of from moe_dispatch, rather than a second copy of the data.
 *   forward:  row r of every product reads X[src_of[r] / k, :] (X [T, d]); Xp is not read.
 *             G, U, H, Yout exactly as moe_expert_fwd would compute them from Xp (same bits).
 *   backward: dH = (dY[src_of[r] / k, :] Wd^T) * topk_w[src_of[r]] row by row, i.e. the weight of the
 *             combine is applied after the product, in fp32, instead of to a rounded copy of the rows;
 *             everything else as moe_expert_bwd.  Xp and dYp = moe_combine_bwd's output are still read,
 *             by the weight gradients only (there the gathered dimension would be the one summed over).
 * Byte offsets into X and dY are 32 bits: T * d * element size must stay below 4 GiB (MOE_EINVAL
 * otherwise).  Workspaces as for moe_expert_fwd / moe_expert_bwd with shared = 0.
 */
int moe_expert_fwd_gather(const moe_shape_t* shape, const int32_t* offsets, const int32_t* src_of, const void* X,
                          const void* Wg, const void* Wu, const void* Wd, void* G, void* U, void* H, void* Yout,
                          void* ws, size_t ws_bytes, void* stream);
int moe_expert_bwd_gather(const moe_shape_t* shape, const int32_t* offsets, const int32_t* src_of, const void* Xp,
                          const void* Wg, const void* Wu, const void* Wd, const void* G, const void* U,
                          const void* H, const void* dY, const float* topk_w, const void* dYp, void* dXp,
                          int32_t* active_ids, int32_t* n_active, void* dWg_c, void* dWu_c, void* dWd_c, void* ws,
                          size_t ws_bytes, void* stream);

/*
 * moe_combine -- the weighted sum of Eq. 3:
 *   Y[t, :] = Yadd[t, :] + sum_j topk_w[t, j] * Yp[row_of[t*k + j], :]
 * accumulated in fp32 and rounded once.  topk_w == NULL means unit weights (this is then the
 * adjoint of the row copy of moe_dispatch, used for dX); Yadd == NULL means no added term
 * (Yadd carries the shared experts' output).  Y may not alias Yp; Y may alias Yadd.
 */
int moe_combine(const moe_shape_t* shape, const void* Yp, const int32_t* row_of, const float* topk_w,
                const void* Yadd, void* Y, void* stream);

/*
 * moe_combine_bwd -- backward of moe_combine with respect to Yp and the weights:
 *   dYp[row_of[a], :] = topk_w[a] * dY[t, :];   dw[a] = <dY[t, :], Yp[row_of[a], :]>,  a = t*k + j.
 *   dY [T, d];  Yp [T*k, d];  dYp [T*k, d] out;  dw [T, k] f32 out
 */
int moe_combine_bwd(const moe_shape_t* shape, const void* dY, const void* Yp, const int32_t* row_of,
                    const float* topk_w, void* dYp, float* dw, void* stream);

/*
 * Per-kernel timing for benchmarks (not part of the hot path; off by default).
 * moe_profile_enable(1) clears earlier records and makes every later kernel launch of this
 * library be bracketed by two HIP events on the launch's own stream; moe_profile_enable(0)
 * stops recording.  moe_profile_report waits for the recorded events and writes one line per
 * kernel label, "<label> <launches> <total milliseconds>\n", into the HOST buffer `buf`
 * (truncated to buf_bytes, always NUL-terminated); it returns the size needed for the whole
 * report.  Not thread-safe against concurrent launches.
 */
int moe_profile_enable(int on);
size_t moe_profile_report(char* buf, size_t buf_bytes);

/*
 * moe_copy_probe -- measurement aid, not part of the hot path: one plain copy kernel
 * (copy_probe_kernel) moving `bytes` bytes from the device buffer `src` to the device buffer
 * `dst` (both 16-byte aligned, bytes a positive multiple of 16, no overlap).  It reads and
 * writes exactly `bytes` bytes of HBM, so a profiler's memory counters for this launch give the
 * factor that converts counter units into bytes for the other kernels of the same run.
 */
int moe_copy_probe(const void* src, void* dst, size_t bytes, void* stream);

/*
 * moe_mfma_probe -- measurement aid, not part of the hot path: a register-resident matrix loop
 * (mfma_probe_kernel).  n_blocks blocks of four wavefronts each issue `iters` rounds of 16 independent
 * v_mfma_f32_32x32x16_bf16 (all 256 accumulator registers in use, one wavefront per SIMD, no loads, no
 * LDS).  Its rate is what the matrix pipe sustains at the clock the chip holds under matrix load: the
 * measured ceiling beside the published 2.5 PFLOP/s.
 *   sink       device buffer of n_blocks * 256 floats (never written in practice; keeps the loop alive)
 *   flops_out  host pointer or NULL: receives the FLOPs of the launch, n_blocks * 4 * iters * 16 * 32768
 */
int moe_mfma_probe(int32_t n_blocks, int32_t iters, float* sink, double* flops_out, void* stream);

/*
 * Host-side planners of the paper.  Every pointer below is HOST memory; nothing here touches the
 * GPU.  E experts, D devices; devices n*dpn .. n*dpn + dpn - 1 form node n (D a multiple of dpn).
 * A placement is an [E, D] matrix of bytes: nonzero = device d holds the parameters of expert e.
 * All calls return MOE_OK or MOE_EINVAL (bad sizes, null pointers, negative or NaN loads,
 * negative token counts, an expert held by no device); outputs are then unspecified.
 *
 * moe_plan_overlap_degree -- t = floor(T_attn * bw / Psi): the expert chunks of Psi bytes that a link
 *   of bandwidth bw absorbs within the attention window T_attn (Section 4.2, after Algorithm 1);
 *   clipped to INT32_MAX.
 * moe_plan_predict_load -- the expert load estimate of Section 4.2: mean of the last min(w, n_iters)
 *   rows of history [n_iters, E] (oldest first; the paper uses w = 5) into F [E].
 * moe_plan_materialize -- Algorithm 1 (Sparse Materialization): from the shard placement P, the
 *   loads F [E] (>= 0), the overlap degree t and the budget m of ephemeral replicas per device to
 *   the plan P_out [E, D], a superset of P (P_out may be P).  t <- min(t, E), m <- min(m, t); the
 *   top-t experts by load (descending, equal loads by ascending id) are candidates.  t <= m: each of
 *   them goes to every device.  Otherwise, in descending load, expert e receives
 *   n = max(1, floor(D m F[e] / sum of the top-t loads)) new replicas (0 if all those loads are 0;
 *   at most one replica per device), placed one at a time on the device that lacks e, has a free
 *   slot, and comes first by (its node already holds e, most free slots, lowest device id) -- the
 *   paper names these two sub-steps without defining them; this is the reading taken.
 * moe_plan_dispatch -- Algorithm 3 (Topology-aware Token Dispatching): from the placement Pm and
 *   the token assignment T [E, D] (tokens of device d routed to expert e) to the plan
 *   R [E, D, D], R[e, d, d2] = tokens of device d sent to expert e on device d2: everything stays
 *   on d when d holds e; otherwise it is split evenly over the holders in d's node if there are
 *   any, else over all holders (floor(x / n) each, one more to the first x mod n holders in
 *   ascending device id).
 */
int moe_plan_overlap_degree(double t_attn, double bw, double psi, int32_t* t_out);
int moe_plan_predict_load(const double* history, int32_t n_iters, int32_t E, int32_t w, double* F);
int moe_plan_materialize(int32_t E, int32_t D, int32_t dpn, const uint8_t* P, const double* F, int32_t t, int32_t m,
                         uint8_t* P_out);
int moe_plan_dispatch(int32_t E, int32_t D, int32_t dpn, const uint8_t* Pm, const int32_t* T, int32_t* R);

#ifdef __cplusplus
}
#endif
#endif /* MOE_HIP_H */
