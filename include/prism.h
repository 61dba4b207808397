/*
 * prism.h -- C ABI of libprism: one edge server's placement-aware MoE layer
 * forward on one AMD MI355X (gfx950), as hand-written HIP kernels.
 *
 * Paper: Prism (arXiv 2508.12851), Sec. III-A (system architecture: a server's
 * gating network picks a token's experts wherever they are hosted, the hosted
 * ones run on that server, the outputs are summed, and the picks are reported
 * to the global scheduler) and Sec. III-B (activation frequency f_n^l(e),
 * placement z_{n,g}^e, indicator 1_remote(n,e), proxy objective Eq. 2).
 *
 * The paper fixes the roles of the steps, not their formulas; this library
 * uses the standard top-k softmax gating and bias-free SwiGLU experts of the
 * two model families the paper evaluates (Sec. IV):
 *
 *   logit[t,e] = fl32( sum_h x[t,h] * W_r[e,h] ) + bias[row(t), e]
 *                (the sum is accumulated in fp64 and rounded once to fp32;
 *                 the fp32 bias is added in fp32)
 *   top-k      : k picks per token by descending logit, lowest expert index
 *                wins ties; slot j holds the j-th pick
 *   gate[t,j]  = exp(l_j - l_0) / sum_j' exp(l_j' - l_0)   (sums to 1; with
 *                gate_mode PRISM_GATES_SOFTMAX_ALL the sum in the denominator
 *                runs over all E experts instead of the k picks)
 *   counts[e]  = number of (t,j) with topk_idx[t,j] == e   (all experts,
 *                hosted or not: the raw f_n^l(e))
 *   local(a)   = local_mask[topk_idx[a]] != 0 for assignment a = t*k + j
 *                (local_mask[e] = [sum_g z_{n,g}^e >= 1] = 1 - 1_remote(n,e))
 *   y_a        = W_down^e ( silu(W_gate^e x_t) * (W_up^e x_t) ),
 *                silu(z) = z / (1 + exp(-z))
 *   out[t]     = sum_{j : local} gate[t,j] * y_(t,j) + sum_s y^shared_(s,t)
 *                (the local partial sum; remote slots are only listed)
 *
 * Conventions
 *   - Every pointer is a DEVICE pointer unless marked "host".  All matrices
 *     are dense row-major.  The caller owns every buffer; the library
 *     allocates nothing on the device and keeps no state between calls.
 *   - Every call only enqueues work on `stream` (a hipStream_t passed as
 *     void*, NULL = the default stream) and never synchronises.  Values that
 *     depend on routing (counts, n_local_remote, remote_bytes, offsets) stay
 *     in device memory; the caller copies them back when it wants them.
 *   - Errors are return codes only.  Arguments are validated on the host
 *     before anything is launched: a NULL required pointer, T < 0, k < 1 or
 *     k > E give PRISM_ERR_INVALID_ARG; sizes outside the compiled limits
 *     give PRISM_ERR_UNSUPPORTED; a workspace smaller than
 *     prism_workspace_bytes() gives PRISM_ERR_WORKSPACE_TOO_SMALL; a failed
 *     kernel launch gives PRISM_ERR_LAUNCH.  T == 0 is PRISM_OK and writes
 *     zero counts / offsets / totals.
 *   - Inputs are assumed finite (not checked).
 *   - Integer outputs are a pure function of the inputs (deterministic).
 *
 * Limits: 1 <= E <= 256, 1 <= k <= 8, k <= E, S <= 16, T*k + S*T < 2^30.
 * H % 8 == 0 for both dtypes; PRISM_BF16 additionally needs H % 64 == 0 and
 * F % 64 == 0 in the FFN, combine and whole-layer calls.  Weight and token
 * matrices must be 16-byte aligned.
 */
#ifndef PRISM_H_
#define PRISM_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  PRISM_OK = 0,
  PRISM_ERR_INVALID_ARG = 1,
  PRISM_ERR_UNSUPPORTED = 2,
  PRISM_ERR_WORKSPACE_TOO_SMALL = 3,
  PRISM_ERR_LAUNCH = 4
} prism_status;

typedef enum { PRISM_F32 = 0, PRISM_BF16 = 1 } prism_dtype;

#define PRISM_MAX_EXPERTS 256
#define PRISM_MAX_TOPK 8
#define PRISM_MAX_SHARED 16

/* Gate values of a token's k picks (the paper leaves the gating function open; the two
 * model families of Sec. IV use one convention each).  The picks themselves, the counts
 * and the split do not depend on it. */
typedef enum {
  PRISM_GATES_RENORMALIZED = 0, /* softmax over the k picked logits: the gates sum to 1 */
  PRISM_GATES_SOFTMAX_ALL = 1   /* the picked entries of the softmax over all E logits */
} prism_gate_mode;

/* Memory layout of every expert weight matrix [rows, cols] (w_gate, w_up: [F,H]; w_down: [H,F]).
 * PRISM_WEIGHTS_TILED (bf16 layers only): tiles of 16 rows x 32 columns, 1 KiB each, stored
 * row-tile major, the rows of a tile 64 bytes apart; element (r, c) lies at byte
 *   ((r / 16) * (cols / 32) + c / 32) * 1024 + (r % 16) * 64 + (c % 32) * 2.
 * A matrix is brought into it once, when the expert is loaded, with prism_pack_weights.  The
 * prefill kernels consume 32 columns of a weight row at a time: from a row-major matrix that is
 * one half of a 128-byte cache line per row, and the L2 delivers the whole line both times;
 * from a tile, every line fetched is used completely.  Results are bit-identical. */
typedef enum { PRISM_WEIGHTS_ROW_MAJOR = 0, PRISM_WEIGHTS_TILED = 1 } prism_weight_layout;

/* Layer description: plain data in HOST memory, passed by const pointer. */
typedef struct {
  int32_t hidden;            /* H */
  int32_t ffn;               /* F */
  int32_t n_experts;         /* E routed experts */
  int32_t top_k;             /* k */
  int32_t n_shared;          /* S always-on shared experts (hosted everywhere) */
  int32_t dtype;             /* prism_dtype of x, every weight matrix, y and out */
  int32_t bias_group_tokens; /* 0: bias row 0 for all tokens; else row = t / this */
  int32_t gate_mode;         /* prism_gate_mode: what the k gate values of a token are */
  int32_t weight_layout;     /* prism_weight_layout of all expert weight matrices */
} prism_layer_desc;

/*
 * Expert weights: a HOST struct holding DEVICE arrays of device pointers.
 * w_gate[e], w_up[e] are [F,H]; w_down[e] is [H,F]; e in [0,E).  An entry may
 * be NULL iff local_mask[e] == 0 (the expert is hosted elsewhere); a hosted
 * expert with a NULL pointer is undefined behaviour.  The shared_* arrays
 * have S entries and may be NULL when S == 0.
 */
typedef struct {
  const void* const* w_gate;
  const void* const* w_up;
  const void* const* w_down;
  const void* const* shared_w_gate;
  const void* const* shared_w_up;
  const void* const* shared_w_down;
} prism_expert_weights;

/* Static text for a status code (host pointer, never NULL). */
const char* prism_status_string(prism_status s);

/*
 * Workspace size in bytes (written to the host variable *bytes) that any
 * entry point below needs for a batch of up to max_tokens tokens of this
 * layer.  The size never shrinks as max_tokens grows, so a workspace sized for
 * the largest batch serves every smaller one.  The workspace must be 256-byte
 * aligned; its contents between calls are irrelevant; two calls that use the
 * same workspace must not overlap in time (run them on one stream, or give
 * each stream its own workspace).
 */
prism_status prism_workspace_bytes(const prism_layer_desc* desc, int32_t max_tokens, size_t* bytes);

/*
 * Gating network + activation statistics (Sec. III-A gating network; Sec.
 * III-B frequency f_n^l(e)).
 *   x            [T,H] layer dtype
 *   w_router     [E,H] layer dtype
 *   router_bias  [G,E] fp32 or NULL; G = 1 or ceil(T / bias_group_tokens)
 *   logits       [T,E] fp32 out, or NULL if not wanted
 *   topk_idx     [T,k] int32 out
 *   topk_gate    [T,k] fp32 out
 *   counts       [E] int32 out, overwritten with this call's counts
 *   counts_accum [E] int64, += this call's counts; or NULL
 */
prism_status prism_route(const prism_layer_desc* desc, const void* x, const void* w_router,
                         const float* router_bias, int32_t T, float* logits, int32_t* topk_idx,
                         float* topk_gate, int32_t* counts, int64_t* counts_accum, void* stream);

/*
 * Placement split (Sec. III-B, indicator 1_remote) and stable bucketing.
 * Assignment a = t*k + j is local iff local_mask[topk_idx[a]] != 0.
 *   local_src      [T*k] int32 out: the local assignments, bucketed by expert
 *                  in ascending expert order, ascending a inside a bucket;
 *                  entries past n_local are not written
 *   local_offsets  [E+1] int32 out: bucket e is local_src[off[e] .. off[e+1])
 *   remote_src / remote_offsets: the same for the assignments whose expert is
 *                  not hosted here (the remote-dispatch list)
 *   n_local_remote [2] int32 out: {n_local, n_remote}
 *   remote_bytes   [2] int64 out: {bytes to send, bytes to receive} =
 *                  n_remote * H * sizeof(element) each (one activation row per
 *                  remote assignment each way: the traffic of a remote call,
 *                  Sec. III-B)
 */
prism_status prism_dispatch(const prism_layer_desc* desc, const int32_t* topk_idx,
                            const uint8_t* local_mask, int32_t T, int32_t* local_src,
                            int32_t* local_offsets, int32_t* remote_src, int32_t* remote_offsets,
                            int32_t* n_local_remote, int64_t* remote_bytes, void* workspace,
                            size_t workspace_bytes, void* stream);

/*
 * Grouped SwiGLU FFN over the locally hosted experts and the shared experts
 * (the local expert execution of Sec. III-A).
 *   y  [T*k + S*T, H] layer dtype out: row r < n_local is the expert output
 *      of assignment local_src[r] (token local_src[r] / k, expert = bucket of
 *      r); rows n_local .. T*k-1 are not written; row T*k + s*T + t is
 *      shared expert s applied to token t.
 * bf16: products accumulate in fp32, silu*up is formed in fp32 and rounded to
 * bf16 once before the down projection, y is rounded to bf16 once.
 */
prism_status prism_expert_ffn(const prism_layer_desc* desc, const void* x,
                              const prism_expert_weights* weights, const int32_t* local_src,
                              const int32_t* local_offsets, int32_t T, void* y, void* workspace,
                              size_t workspace_bytes, void* stream);

/*
 * Gate-weighted aggregation of the local expert outputs (the last step of
 * the layer in Sec. III-A): out[t] = sum over local slots j (ascending) of
 * topk_gate[t,j] * y[row of (t,j)], then + shared rows s = 0..S-1, in fp32,
 * rounded once to the layer dtype.  A token with no local slot and S == 0
 * gets zeros.
 *   out [T,H] layer dtype
 */
prism_status prism_combine(const prism_layer_desc* desc, const void* y, const int32_t* local_src,
                           const int32_t* local_offsets, const float* topk_gate, int32_t T,
                           void* out, void* workspace, size_t workspace_bytes, void* stream);

/*
 * The two ends of the remote call on the requesting server (Sec. III-A: the
 * request to the hosting server and the aggregation of what it returns;
 * Sec. III-B: what travels is the activation).
 *
 * prism_pack_remote gathers the activation rows to ship, in remote-list order:
 *   packed[r] = x[remote_src[r] / k]  for r < remote_offsets[E]
 *   packed [T*k, H] layer dtype (rows past the remote count untouched).
 * Segment remote_offsets[e]..[e+1] of packed is what the server hosting expert
 * e receives; that server runs prism_expert_ffn on it (top_k = 1, no shared
 * experts, local_src = 0..R-1, local_offsets = the received segment sizes).
 *
 * prism_combine_remote adds the returned rows to the local partial sum:
 *   out[t] = out[t] + sum over remote slots j (ascending) of
 *            topk_gate[t,j] * y_remote[row of (t,j) in the remote list]
 * in fp32, rounded once more to the layer dtype; with prism_moe_layer's out it
 * completes the layer (= the layer with every expert hosted, up to rounding).
 *   y_remote [>= R, H] layer dtype, rows in remote-list order;  out [T,H] in/out.
 * The workspace is used for the inverse of the remote list (do not run it
 * concurrently with another call on the same workspace).
 */
prism_status prism_pack_remote(const prism_layer_desc* desc, const void* x, const int32_t* remote_src,
                               const int32_t* remote_offsets, int32_t T, void* packed, void* stream);
prism_status prism_combine_remote(const prism_layer_desc* desc, const void* y_remote,
                                  const int32_t* remote_src, const int32_t* remote_offsets,
                                  const float* topk_gate, int32_t T, void* out, void* workspace,
                                  size_t workspace_bytes, void* stream);

/*
 * The whole layer: route -> dispatch -> expert FFN -> combine, on one stream,
 * with no host synchronisation.  Outputs as in the calls above; local_src,
 * local_offsets, the FFN intermediate and y live in the workspace.
 */
prism_status prism_moe_layer(const prism_layer_desc* desc, const void* x, const void* w_router,
                             const float* router_bias, const prism_expert_weights* weights,
                             const uint8_t* local_mask, int32_t T, void* out, int32_t* topk_idx,
                             float* topk_gate, int32_t* counts, int64_t* counts_accum,
                             int32_t* remote_src, int32_t* remote_offsets,
                             int32_t* n_local_remote, int64_t* remote_bytes, void* workspace,
                             size_t workspace_bytes, void* stream);

/*
 * prism_moe_layer for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The
 * same layer, the same kernels, the same results bit for bit; the scratch memory is a fixed
 * array of PRISM_STATIC_SCRATCH_BYTES that lives in the library's device image (every GPU
 * the process uses holds its own copy until the process ends).  The call allocates and frees
 * nothing, and neither does anything it calls.
 *   - Accepted while prism_workspace_bytes(desc, T) <= PRISM_STATIC_SCRATCH_BYTES (32 MiB:
 *     e.g. decode batches of up to 64 tokens of a 4096 x 14336 layer with 8 experts, 2048
 *     tokens of a 256 x 448 layer); beyond that PRISM_ERR_WORKSPACE_TOO_SMALL, nothing launched.
 *   - The first call on a device looks up that device's address of the array (one
 *     hipGetSymbolAddress; PRISM_ERR_LAUNCH if it fails); make that call outside any capture.
 *   - All calls on one GPU share the one array, which keeps the previous call's contents
 *     (no step of the layer reads scratch it has not written in the same call, so nothing
 *     needs clearing): calls that overlap in time on one GPU -- two streams, two threads --
 *     race on it.  Run them on one stream, or give the others prism_moe_layer and a workspace.
 *   - prism_layer_permutation does not apply (there is no workspace to name).
 * Other arguments, outputs and errors as prism_moe_layer.
 */
#define PRISM_STATIC_SCRATCH_BYTES (32u << 20)
prism_status prism_moe_layer_static(const prism_layer_desc* desc, const void* x, const void* w_router,
                                    const float* router_bias, const prism_expert_weights* weights,
                                    const uint8_t* local_mask, int32_t T, void* out, int32_t* topk_idx,
                                    float* topk_gate, int32_t* counts, int64_t* counts_accum,
                                    int32_t* remote_src, int32_t* remote_offsets,
                                    int32_t* n_local_remote, int64_t* remote_bytes, void* stream);

/*
 * The permutation the placement split of Sec. III-B produced inside the last whole-layer
 * call (prism_moe_layer, prism_moe_layer_traced) that used `workspace` with the same desc
 * and T: that call keeps local_src / local_offsets in the workspace, this one copies them
 * out (device-to-device copies enqueued on `stream`; enqueue it on the layer's stream, or
 * after that call has finished, and before the workspace is used again).
 *   local_src     [T*k] int32 out, as prism_dispatch defines it; entries past n_local
 *                 hold whatever the workspace held
 *   local_offsets [E+1] int32 out
 *   inv           [T*k] int32 out or NULL: row of assignment a in the layer's y, -1 if remote
 * Errors: as the layer call (INVALID_ARG, UNSUPPORTED, WORKSPACE_TOO_SMALL); PRISM_ERR_LAUNCH
 * if a copy cannot be enqueued.
 */
prism_status prism_layer_permutation(const prism_layer_desc* desc, int32_t T, const void* workspace,
                                     size_t workspace_bytes, int32_t* local_src,
                                     int32_t* local_offsets, int32_t* inv, void* stream);

/*
 * prism_moe_layer with stage timing for measurement harnesses.  stage_events
 * is a HOST array of 2 * PRISM_N_STAGES hipEvent_t handles (as void*), or
 * NULL.  For stage s, if stage_events[2s] and stage_events[2s+1] are both
 * non-NULL, the first is recorded on `stream` right before and the second
 * right after that stage's kernels: the router kernel, the dispatch kernels,
 * the gate/up grouped GEMM alone, the down grouped GEMM, the combine kernel.
 * For decode-sized bf16 batches (T <= 64) the work is cut differently: ROUTE
 * is the router GEMM with the hidden dimension split over workgroups,
 * DISPATCH the single-workgroup kernel that finishes the routing, does the
 * placement split and builds the GEMM work lists, and COMBINE also sums the
 * contraction slices of the down projection.  Nothing else differs from
 * prism_moe_layer, which is this call with stage_events == NULL.
 */
#define PRISM_STAGE_ROUTE 0
#define PRISM_STAGE_DISPATCH 1
#define PRISM_STAGE_FFN_UP 2
#define PRISM_STAGE_FFN_DOWN 3
#define PRISM_STAGE_COMBINE 4
#define PRISM_N_STAGES 5
prism_status prism_moe_layer_traced(const prism_layer_desc* desc, const void* x,
                                    const void* w_router, const float* router_bias,
                                    const prism_expert_weights* weights,
                                    const uint8_t* local_mask, int32_t T, void* out,
                                    int32_t* topk_idx, float* topk_gate, int32_t* counts,
                                    int64_t* counts_accum, int32_t* remote_src,
                                    int32_t* remote_offsets, int32_t* n_local_remote,
                                    int64_t* remote_bytes, void* workspace, size_t workspace_bytes,
                                    void* stream, void* const* stage_events);

/*
 * Re-lays a row-major bf16 matrix [rows, cols] into PRISM_WEIGHTS_TILED (see
 * prism_weight_layout).  rows must be a multiple of 16, cols of 32; src and dst are device
 * buffers of rows * cols * 2 bytes, 16-byte aligned, and must not overlap.  Enqueues one
 * kernel on `stream`.  Errors: PRISM_ERR_INVALID_ARG (NULL, sizes < 1, misaligned),
 * PRISM_ERR_UNSUPPORTED (rows not a multiple of 16, cols not of 32, or the matrix is 4 GiB or more).
 */
prism_status prism_pack_weights(const void* src, int32_t rows, int32_t cols, void* dst, void* stream);

/*
 * Debug helper, NOT asynchronous: copies the pointer tables and the mask back
 * to the host (blocking copies on the default stream) and checks what the fast
 * path assumes without checking: every hosted expert (local_mask[e] != 0) and
 * every shared expert has three non-NULL, 16-byte aligned weight pointers.
 * Returns PRISM_OK, or PRISM_ERR_INVALID_ARG with *bad_expert (host, may be
 * NULL) set to the first offending routed expert, or to E + s for shared
 * expert s.  PRISM_ERR_LAUNCH if a copy fails.
 */
prism_status prism_debug_check_weights(const prism_layer_desc* desc,
                                       const prism_expert_weights* weights,
                                       const uint8_t* local_mask, int32_t* bad_expert);

/*
 * Measured ceilings for measurement harnesses (not steps of the method).  Both
 * calls only enqueue one kernel on `stream`; the caller times it.
 *
 * prism_ceiling_mfma_bf16: n_workgroups workgroups of 256 threads each run
 * `iters` iterations of 8 independent v_mfma_f32_32x32x16_bf16 per wavefront.
 *   operands  device, 16-byte aligned, n_workgroups * 256 * 2 vectors of 8
 *             bf16: thread i multiplies vector 2i by vector 2i+1 (the clock
 *             the chip sustains depends on these values)
 *   out       device, n_workgroups * 256 floats (written, keeps the loop alive)
 *   flop      host, receives the floating-point operations of the launch
 *
 * prism_ceiling_hbm_read: n_workgroups workgroups of 256 threads read `bytes`
 * bytes (a multiple of 16 is read; use a buffer larger than the 256 MB
 * last-level cache) with 16-byte loads, grid-strided.  Thread i stores the xor
 * of the vectors it read to out[i] only when that xor is not zero, so an
 * all-zero source is read without any write traffic.
 *   src  device, 16-byte aligned;  out  device, n_workgroups * 256 * 16 bytes
 * Errors: PRISM_ERR_INVALID_ARG for NULL or misaligned pointers, counts < 1.
 */
/*
 * prism_ceiling_hbm_read_pattern: the streaming read with its access pattern as arguments,
 * for finding the pattern this machine's memory system serves fastest.  The first
 * floor(bytes / span_bytes) spans of src are read; workgroup b (256 threads) takes spans
 * b, b + n_workgroups, ... and walks each with loads_in_flight (2, 4, 8 or 16) loads of 16
 * bytes per thread in flight.  mode 0: loads into registers; 1: direct-to-LDS loads, 1 KiB per
 * wavefront and instruction (what the grouped GEMM's operand rings issue); 2: loads marked
 * non-temporal; 3: direct-to-LDS loads marked non-temporal.  span_bytes must be a multiple of 4096 * loads_in_flight, at most 2 GiB.
 *   bytes_read  host, receives the bytes the launch reads;  out  device, n_workgroups * 4096 bytes
 * Errors: INVALID_ARG (NULL, misaligned, counts < 1, unknown mode, fewer bytes than one
 * span), UNSUPPORTED (loads_in_flight or span_bytes outside the above).
 */
prism_status prism_ceiling_hbm_read_pattern(const void* src, size_t bytes, void* out, int32_t n_workgroups,
                                            int32_t loads_in_flight, size_t span_bytes, int32_t mode,
                                            size_t* bytes_read, void* stream);
prism_status prism_ceiling_mfma_bf16(const void* operands, float* out, int32_t n_workgroups,
                                     int32_t iters, double* flop, void* stream);
prism_status prism_ceiling_hbm_read(const void* src, size_t bytes, void* out, int32_t n_workgroups,
                                    void* stream);

#ifdef __cplusplus
}
#endif
#endif /* PRISM_H_ */
