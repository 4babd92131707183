/*
 * oea.h - C ABI of the MI355X (gfx950) decode-time MoE layer with Opportunistic Expert
 * Activation (OEA, arxiv 2511.02237).
 *
 * Conventions for every entry point
 *   - Pointers are DEVICE pointers (HBM of the current HIP device) unless the name starts with h_.
 *   - The caller owns every buffer; the library allocates no device memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only enqueue
 *     work and return; results are valid once the caller has synchronised the stream.  Nothing
 *     is read back to the host, so a call sequence can be captured into a HIP graph.  The one
 *     exception is oea_workspace_check, which synchronises the stream and reads one word back.
 *   - Return value: OEA_OK (0) or a negative oea_status.  Every argument check comes before the
 *     first enqueue, so a call refused for its arguments has enqueued nothing; OEA_ERR_HIP can
 *     come from a launch or copy in the middle of a call, after earlier kernels were enqueued.
 *   - The library keeps no state between calls except what it looks up once per device (compute
 *     unit count, kernel attributes) and the built-in scratch of moe_decode_static.
 *   - All matrices are row-major, expert ids are 0-based (the paper counts from 1).
 *   - Non-finite router logits give unspecified routing, but never an out-of-range index.
 */
#ifndef OEA_H_
#define OEA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  OEA_OK = 0,
  OEA_ERR_NULL = -1,      /* a required pointer is NULL */
  OEA_ERR_SHAPE = -2,     /* B<1, N<1, d or I not a positive multiple of 8, or above the limits below */
  OEA_ERR_K = -3,         /* not (1 <= k0 <= k <= min(N, OEA_MAX_K)) */
  OEA_ERR_ALIGN = -4,     /* x / weight / workspace pointer not 16-byte aligned */
  OEA_ERR_WORKSPACE = -5, /* workspace_bytes < oea_workspace_bytes(...) */
  OEA_ERR_DTYPE = -6,     /* unknown oea_dtype */
  OEA_ERR_HIP = -7,       /* a HIP runtime call failed (no device, launch failure) */
  OEA_ERR_TIMEOUT = -8,   /* oea_workspace_check: a bounded wait inside a kernel gave up */
  OEA_ERR_LIMIT = -9,     /* moe_decode_static: oea_workspace_bytes(...) > OEA_STATIC_SCRATCH_BYTES */
  OEA_ERR_WORKSPACE_STATE = -10 /* oea_workspace_check: the workspace was not prepared by
                                   oea_workspace_init (or has been overwritten since) */
} oea_status;

/* storage type of x, W_router, W_gate, W_up, W_down (all the same).  Entry points take it as a
 * plain int `dt` and answer any other value with OEA_ERR_DTYPE. */
typedef enum { OEA_F32 = 0, OEA_BF16 = 1 } oea_dtype;

#define OEA_MAX_N 512  /* experts */
#define OEA_MAX_K 32   /* experts per token */
#define OEA_MAX_B 1024 /* tokens per decode batch */
#define OEA_MAX_D 8192 /* embedding dimension and expert hidden dimension */
#define OEA_MAX_POSITIONS 65535 /* decode positions per oea_route_batched call */
#define OEA_STATIC_SCRATCH_BYTES 8388608 /* device scratch built into the library for moe_decode_static */

/* Host, pure.  Static text for a status code. */
const char *oea_status_string(int status);

/* Host, pure.  Bytes of device workspace moe_decode needs for these sizes (0 on bad sizes). */
size_t oea_workspace_bytes(int B, int d, int N, int I, int k);

/* Host, pure.  The same for calls with oea_decode_ex.deterministic set (adds B*k*d floats). */
size_t oea_workspace_bytes_deterministic(int B, int d, int N, int I, int k);

/*
 * Prepare a workspace: enqueues a kernel that zeroes its control words and marks it as prepared.
 * Call once after allocating (or re-using for something else) a workspace, before the first
 * moe_decode on it.  Each moe_decode leaves the words it synchronises through zero again, so one
 * call serves any number of layers.  A layer enqueued on a workspace without the mark does not
 * wait for anything: its kernels return early, `out` is undefined (zero on the three-kernel
 * path) and oea_workspace_check reports OEA_ERR_WORKSPACE_STATE.  The workspace also carries a small load-balancing state from call to call (a
 * speed estimate per workgroup that steers how the weight rows are shared out); it changes
 * timing only, and the order of the floating-point additions into `out`.
 */
int oea_workspace_init(void *workspace, size_t workspace_bytes, void *stream);

/*
 * OEA routing of one decode batch from given router logits: Algorithm 1 of the paper
 * (Phase 1: each token keeps its k0 best experts; Phase 2: in rank order it adds experts that are
 * in the union of all tokens' Phase-1 sets, until it holds k), followed by the weighting of
 * Section 3.2 "Weighting after rerouting" (softmax scores renormalised over the final set, Eq. 1).
 * k0 == k is the unmodified top-k router.
 *
 *   router_logits [B,N] fp32   router pre-activations; ranking is by descending logit, equal
 *                              logits by ascending expert id (-0.0 == +0.0)
 *   expert_idx    [B,k] int32  S_i in rank order, -1 in unused slots
 *   gate_w        [B,k] fp32   weights, 0 in unused slots, each row sums to 1
 *   n_sel         [B]   int32  |S_i| = min(k, T)
 *   active_list   [N]   int32  the union S^base, ascending; entries >= T are -1
 *   n_active      [1]   int32  T = |S^base|
 * Limits: N <= OEA_MAX_N, k <= OEA_MAX_K, B <= OEA_MAX_B.
 */
int oea_route(const float *router_logits, int B, int N, int k, int k0, int32_t *expert_idx,
              float *gate_w, int32_t *n_sel, int32_t *active_list, int32_t *n_active,
              void *stream);

/*
 * oea_route for L independent decode positions in one launch (Section 4.1, "Methodology": routing
 * runs only within a decode step, and the paper's cross-entropy evaluation routes all positions of
 * its sequences in parallel this way).  Position l uses rows [l*B, (l+1)*B) of the logits and nothing else.
 *   router_logits [L,B,N]; token_mask [L,B] uint8 or NULL (0 = padding token);
 *   expert_idx, gate_w [L,B,k]; n_sel [L,B]; active_list [L,N]; n_active [L].
 * Limits as oea_route, 1 <= L <= OEA_MAX_POSITIONS.
 */
int oea_route_batched(const float *router_logits, const uint8_t *token_mask, int L, int B, int N,
                      int k, int k0, int32_t *expert_idx, float *gate_w, int32_t *n_sel,
                      int32_t *active_list, int32_t *n_active, void *stream);

/*
 * General OEA routing (Algorithm 2 of the paper, Section 3.2 "The Proposed Routing Algorithm",
 * paragraphs "Phase 1: Baseline expert selection" and "Phase 2: Opportunistic piggybacking"): as
 * oea_route, with
 *   - a top-p cut of the baseline: n_i = min(k0, t_i), where t_i is the smallest t such that the t
 *     best experts of token i hold softmax mass >= p (sorted cumulative sum; p = 1 switches the
 *     cut off, which is how the paper's experiments run it),
 *   - k_max, the number of experts a token may hold after piggybacking (a baseline that is already
 *     larger is kept as it is), and
 *   - max_p: only experts among the token's max_p best-ranked ones are piggybacked.
 * p = 1, k_max = k, max_p = N gives exactly oea_route(k, k0).
 *
 *   token_mask  [B] uint8 or NULL   0 = padding token (selects nothing, adds nothing to the union)
 *   expert_idx  [B,kw] int32, gate_w [B,kw] fp32 with kw = max(k0, k_max); layout as in oea_route
 *   n_base      [B] int32 or NULL   n_i, the size of each token's baseline
 * The top-p comparison is made on fp64 sums of fp64 softmax values.
 * Errors: OEA_ERR_K unless 1 <= k0 <= N, 1 <= k_max <= N, max(k0,k_max) <= OEA_MAX_K,
 * 1 <= max_p <= N and 0 < p <= 1.
 */
int oea_route_general(const float *router_logits, const uint8_t *token_mask, int B, int N, int k0,
                      double p, int k_max, int max_p, int32_t *expert_idx, float *gate_w,
                      int32_t *n_sel, int32_t *n_base, int32_t *active_list, int32_t *n_active,
                      void *stream);

/*
 * One decode-time MoE layer (Section 2, Eq. 1) with OEA routing (Algorithm 1):
 *   logits = x W_router^T -> routing as in oea_route -> out[i] = sum_{e in S_i} g_{i,e} E_e(x_i),
 *   E_e(x) = W_down[e] ( silu(W_gate[e] x) * (W_up[e] x) )      (Section 4: SwiGLU expert)
 * Only the T experts of the union are read from memory, each once.
 *
 *   x        [B,d]    dt      token embeddings
 *   W_router [N,d]    dt
 *   W_gate   [N,I,d]  dt      per expert [I,d]: row j produces hidden unit j
 *   W_up     [N,I,d]  dt
 *   W_down   [N,d,I]  dt      per expert [d,I]: row c produces output coordinate c
 *   out      [B,d]    fp32    overwritten.  The weighted sum over a token's experts is accumulated with
 *                             fp32 atomics in arrival order (results of two calls can differ in the last
 *                             places) unless oea_decode_ex.deterministic asks for a fixed order
 *   workspace         device scratch of >= oea_workspace_bytes(B,d,N,I,k) bytes, 16-byte aligned,
 *                     prepared once by oea_workspace_init.  Two calls that share a workspace must
 *                     be ordered on the same stream.
 * For the Qwen3-30B-A3B and Qwen3-235B-A22B layer shapes (bf16, N <= 128, k <= 16, B <= 128) the
 * whole layer runs as ONE persistent kernel with one workgroup per compute unit, one grid-wide
 * barrier and per-expert completion counters; it expects the device to itself while it runs (a
 * workgroup that cannot be placed delays the others; every wait is bounded, after about a second
 * the call gives up, its output is undefined and oea_workspace_check reports OEA_ERR_TIMEOUT).
 * A caller that runs other kernels beside the layer (a second stream) sets
 * oea_decode_ex.cooperative, which makes co-residency the runtime's guarantee.  Still larger batches run as
 * three kernels (router + routing, gate/up stage, down stage) with the expert stages on the matrix
 * cores (bf16, d and I multiples of 256: an expert then serves 16 and more tokens and the
 * arithmetic per pair, Eq. 2's second term, would bound the vector ALUs); every other shape, and fp32
 * storage, runs as three kernels with dot-product expert kernels.
 * Arithmetic: router logits are accumulated in fp64 and rounded once to fp32; expert mat-vecs
 * multiply in the storage type and accumulate in fp32; with bf16 storage the hidden vector is
 * rounded to bf16 between the two mat-vecs (as a bf16 model does).
 * Limits: d, I multiples of 8 and <= OEA_MAX_D; N, k, B as for oea_route.
 */
int moe_decode(const void *x, const void *W_router, const void *W_gate, const void *W_up,
               const void *W_down, float *out, int B, int d, int N, int I, int k, int k0,
               int dt, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Host, synchronises `stream`.  The single-kernel layer waits for other workgroups in a few places;
 * every such wait is bounded, and a workgroup whose wait runs out records that in the workspace
 * and goes on (the call still returns, with undefined output).  This call reports it: OEA_OK if no
 * wait has given up on this workspace since oea_workspace_init, else OEA_ERR_TIMEOUT (the record
 * stays until the workspace is initialised again); OEA_ERR_WORKSPACE_STATE if the workspace does
 * not carry the mark of oea_workspace_init at all.  Callers that cannot rule out sharing the
 * device with other kernels call it after a batch of layers.
 */
int oea_workspace_check(const void *workspace, size_t workspace_bytes, void *stream);

/* Optional inputs and taps for moe_decode_ex; every pointer may be NULL. */
typedef struct {
  const float *router_bias;   /* [N] fp32 added to the logits (synthetic skewed-popularity workload) */
  const uint8_t *token_mask;  /* [B] 0 = padding token: selects nothing, adds nothing to the union,
                                 out row = 0 (Section 6, "A note on padding") */
  float *logits_out;          /* [B,N] the fp32 logits the routing was taken on */
  int32_t *expert_idx_out;    /* [B,k] */
  float *gate_w_out;          /* [B,k] */
  int32_t *n_sel_out;         /* [B]   */
  int32_t *active_list_out;   /* [N]   */
  int32_t *n_active_out;      /* [1]   */
  double top_p;               /* general OEA (Algorithm 2): top-p cut of the baseline; 0 or >= 1 = off
                                 (negative or NaN: OEA_ERR_K) */
  int32_t max_p;              /* general OEA: piggyback only among the max_p best ranks; 0 or >= N = off
                                 (negative: OEA_ERR_K).
                                 With either set, k plays the role of k_max.  Where the single-kernel layer
                                 applies (see moe_decode) the general routing runs inside that kernel. */
  int32_t deterministic;      /* non-zero: Eq. 1's sum over the selected experts is taken in slot order by
                                 one thread per output element (a last small kernel), instead of with
                                 floating-point atomics in arrival order: `out` is then bit-identical from
                                 call to call.  Needs oea_workspace_bytes_deterministic(...) bytes of
                                 workspace; costs one more kernel launch (about 5 us at B=16). */
  int32_t cooperative;        /* non-zero: the single persistent kernel is launched as a cooperative
                                 launch, so the runtime guarantees that all its workgroups are resident
                                 together or refuses the launch (OEA_ERR_HIP) - for callers that share
                                 the device with other work.  Costs about 18 us per call on MI355X. */
} oea_decode_ex;

/* moe_decode with the extras above (ex == NULL behaves as moe_decode). */
int moe_decode_ex(const void *x, const void *W_router, const void *W_gate, const void *W_up,
                  const void *W_down, float *out, int B, int d, int N, int I, int k, int k0,
                  int dt, void *workspace, size_t workspace_bytes, void *stream,
                  const oea_decode_ex *ex);

/*
 * moe_decode_ex for callers that cannot allocate device memory or pass a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same layer, same kernels,
 * same arguments and results as moe_decode_ex (ex may be NULL), but the workspace is a device
 * array built into the library (OEA_STATIC_SCRATCH_BYTES per GPU the library runs on, held until
 * the process ends) instead of an argument.  The call allocates nothing and frees nothing.
 *   - Sizes whose oea_workspace_bytes(B,d,N,I,k) exceeds OEA_STATIC_SCRATCH_BYTES are rejected
 *     with OEA_ERR_LIMIT before anything is enqueued (8 MiB covers B <= 128 at both Qwen3 shapes).
 *   - Every call on a GPU shares that GPU's array and finds the previous call's contents in it
 *     (what has to start at zero is cleared by the kernels themselves): calls on one GPU must be
 *     ordered on one stream; calls that overlap on one GPU race.
 *   - The first call on each GPU also enqueues the kernel that prepares the array (the work of
 *     oea_workspace_init); make that call outside stream capture.
 *   - oea_workspace_check has no counterpart here; callers that share the device with other
 *     kernels use moe_decode_ex with a workspace of their own.
 */
int moe_decode_static(const void *x, const void *W_router, const void *W_gate, const void *W_up,
                      const void *W_down, float *out, int B, int d, int N, int I, int k, int k0,
                      int dt, void *stream, const oea_decode_ex *ex);

#ifdef __cplusplus
}
#endif
#endif /* OEA_H_ */
