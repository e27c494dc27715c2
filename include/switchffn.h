/*
 * switchffn.h -- C ABI of the MI355X (gfx950) Switch FFN layer library.
 *
 * The layer is the sparse feed-forward layer of the Switch Transformer
 * (arXiv 2101.03961): a top-1 router, capacity-limited dispatch of tokens to
 * experts, one ReLU FFN per expert, a gate-weighted combine, and the
 * load-balancing auxiliary loss, forward and backward.  The T tokens form
 * n_groups routing groups of consecutive tokens (the appendix listing's
 * num_cores); by default one group holds them all.
 *
 * General rules
 *   - Every tensor pointer is a DEVICE pointer (HBM) unless a comment says
 *     "host".  The caller owns all memory; the library never allocates, frees
 *     or keeps a pointer after the call's work has run.
 *   - Tensors are dense, row-major, with the shapes given below; base pointers
 *     must be 16-byte aligned.
 *   - Calls are asynchronous: work is queued on `hip_stream` (a hipStream_t
 *     passed as void*; NULL = the default stream) and the call returns without
 *     synchronising.
 *   - Every function returns SW_OK (0) or a negative sw_status.  Errors are
 *     detected on the host before anything is launched; nothing is thrown
 *     across the ABI.  Inputs must be finite (NaN/Inf behaviour unspecified).
 *   - Gradients are overwritten, not accumulated.
 *   - The library keeps no state between calls apart from what the workspace holds and a
 *     few values it looks up once per device (std::call_once: kernel attributes, the number of
 *     compute units, the address of the static scratch array); with profiling off, calls
 *     from several host threads may run at once if each has its own workspace, outputs and
 *     stream.  Work runs on the device that is current when the call is made.
 *   - An empty batch (T = 0) is legal: forward writes expert_counts = 0 and
 *     aux_loss = 0 (both fractions of Eq. 4 are empty sums), backward writes
 *     zeros to dW_r, db_r, dW_in, dW_out; the per-token arguments and the
 *     workspace are not touched and may be NULL.
 *   - act_dtype SW_BF16: x, W_in, W_out, y, dy, dx, dW_in, dW_out are bfloat16
 *     (d_model and d_ff must be multiples of 8); products are accumulated in
 *     fp32 and rounded once (nearest-even) at each store.  SW_F32: the same
 *     tensors are fp32.  The router (W_r, b_r, logits, softmax, gate, aux loss,
 *     dW_r, db_r) is fp32 in both cases ("selective precision", Sec. 2.4).
 *     With bf16 tokens and E a multiple of 4 its contractions run on the
 *     matrix cores (fp32 weights as exact sums of bf16 terms); otherwise on the
 *     vector ALUs, with the same results to rounding and several times slower.
 */
#ifndef SWITCHFFN_H
#define SWITCHFFN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { SW_F32 = 0, SW_BF16 = 1 } sw_dtype;

/* Expert FFN variants.  SW_FFN_RELU: ReLU(x W_in) W_out, W_in [E, d_model, d_ff] (Sec. 5's
 * review of the FFN layer).  SW_FFN_GEGLU: the FFN_GEGLU of the model tables (App. "Switch
 * models"): the expansion matrix is replaced by two, combined as GELU(x W_g) * (x W_l) with
 * the exact GELU(u) = u Phi(u); W_in is then [E, d_model, 2 d_ff] with the d_ff gate columns
 * W_g first and the d_ff linear columns W_l after them, and dW_in has the same shape. */
typedef enum { SW_FFN_RELU = 0, SW_FFN_GEGLU = 1 } sw_ffn_kind;

typedef enum {
    SW_OK = 0,
    SW_ERR_NULL = -1,      /* a required pointer is NULL                         */
    SW_ERR_SHAPE = -2,     /* T, d_model, d_ff, E, n_groups out of range; rows not whole
                              16-byte chunks; bf16: an expert's weight matrix or its
                              slots x max(d_model, d_ff) activations reach 2 GB       */
    SW_ERR_VALUE = -3,     /* capacity_factor not finite or <= 0, alpha not finite,
                              expert_dropout or jitter_eps outside [0, 1), ntlb_rounds
                              outside 0 .. 16, unknown bits in flags                */
    SW_ERR_DTYPE = -4,     /* act_dtype is neither SW_F32 nor SW_BF16, or ffn_kind
                              is not a sw_ffn_kind                               */
    SW_ERR_WORKSPACE = -5, /* workspace NULL, misaligned or too small            */
    SW_ERR_ALIGN = -6,     /* a tensor pointer is not 16-byte aligned            */
    SW_ERR_LAUNCH = -7,    /* the HIP runtime refused a launch (see hipGetLastError) */
    SW_ERR_STATE = -8,     /* profiling calls out of order                       */
    SW_ERR_STATIC_LIMIT = -9 /* switch_forward_static: the configuration's workspace
                              exceeds SW_STATIC_SCRATCH_BYTES                      */
} sw_status;

/* Layer description (host struct, passed by pointer, copied by the callee). */
typedef struct {
    int64_t T;               /* tokens in the batch (0 .. 2^31 - 1)                 */
    int64_t d_model;         /* token width                                         */
    int64_t d_ff;            /* expert hidden width                                 */
    int64_t E;               /* number of experts (1 .. 4096)                       */
    double capacity_factor;  /* > 0; Eq. 3                                          */
    float alpha;             /* auxiliary-loss coefficient (Sec. 2.2; paper: 1e-2)  */
    int32_t act_dtype;       /* sw_dtype of activations and expert weights          */
    int32_t ffn_kind;        /* sw_ffn_kind; 0 = the ReLU FFN                       */
    int64_t n_groups;        /* routing groups of T / n_groups consecutive tokens:
                                capacity (Eq. 3 with the group's token count),
                                position_in_expert and the two fractions of the loss
                                are taken per group, the loss is the mean over groups,
                                the experts are shared.  Must divide T; 0 is read as 1 */
    /* Training-time noise, both off at 0.  The draws are a pure function of (seed,
       element): see "Random draws" below.  Forward and backward of one step must be
       given the same three values; change the seed from step to step. */
    float expert_dropout;    /* Sec. 2.4: rate in [0, 1) at which the hidden activations
                                ReLU(x W_in) of every expert are zeroed; survivors are
                                scaled by 1 / (1 - rate).  Takes effect rounded down to a
                                multiple of 2^-16                                     */
    float jitter_eps;        /* App. C input jitter: the router (and only the router)
                                sees x[t][k] * m, m uniform in [1 - eps, 1 + eps);
                                eps in [0, 1)                                         */
    uint64_t seed;
    int32_t ntlb_rounds;     /* No-Token-Left-Behind (App. B): re-routing stages after the
                                Switch routing, 0 (off) .. 16.  In each stage the tokens
                                still without a slot ask their next-best expert (by logit;
                                equal logits: lower index first) for the capacity it has
                                left, in sequence order inside the routing group.       */
    int32_t flags;           /* 0, or SW_FLAG_FUSED_DISPATCH; other bits are refused
                                with SW_ERR_VALUE                                       */
} switch_config;

/* The dispatch and the combine of Sec. 5.4 are passes of their own over an expert-major copy of
 * the tokens.  With this flag a bf16 layer (whose x is below 2 GB; otherwise the flag has no
 * effect) runs them inside the expert GEMMs instead: token rows are gathered by the operand
 * loads, output rows are written to their tokens by the second GEMM's epilogue.  That needs
 * about 4 % less memory traffic and no expert-major copies of x and dy, and takes 1-2 % longer
 * at the Switch-Base shape.  Same results up to rounding (the gate is applied at a different
 * place). */
#define SW_FLAG_FUSED_DISPATCH 1

/*
 * Random draws.  Element number idx (a 32-bit integer that wraps) of stream s gets the
 * 32 bits
 *     z = (idx ^ seed_lo) * 0x9E3779B1;  z ^= z >> 15;
 *     z = (z + seed_hi + s * 0x7F4A7C15) * 0x85EBCA77;  z ^= z >> 13;
 *     z *= 0xC2B2AE3D;  z ^= z >> 16;            (all arithmetic modulo 2^32)
 * with seed_lo / seed_hi the two halves of seed.
 *   jitter  (s = 1, idx = t * d_model + k):  m = fma(2 eps, (z >> 8) * 2^-24, 1 - eps) in fp32
 *   dropout (s = 2):  hidden unit j of token t (the token -- not its slot) is element
 *           i = t * d_ff + j; it takes 16 bits of the z drawn for idx = i / 2 -- z & 0xFFFF if
 *           i is even, z >> 16 if odd -- and is zeroed iff they are < thr = floor(rate * 2^16);
 *           survivors are scaled by 2^16 / (2^16 - thr)
 * With jitter_eps > 0 and bf16 tokens the workspace also holds x * m as three bf16 planes
 * (6 * T * d_model bytes, d_model rounded up to a multiple of 32).
 */

/* Expert capacity, Eq. 3, rounded down:
 *   capacity = floor((double)(T / n_groups) / (double)E * capacity_factor)
 * -- slots per expert and routing group.
 * Zero is legal (every token is dropped).  Host only. */
int switch_capacity(const switch_config *cfg, int64_t *capacity_out /* host */);

/* Bytes of device workspace that switch_forward/switch_backward need for this
 * configuration (saved activations, routing tables, gradient staging).  Host
 * only.  The workspace must be 256-byte aligned. */
int switch_workspace_size(const switch_config *cfg, size_t *bytes_out /* host */);

/*
 * Forward pass (Sec. 2.1, 2.2; Fig. 2; Eqs. 1, 3-6).
 *   logits h = x W_r (+ b_r), fp32;  p = softmax(h)                    (Eq. 1)
 *   expert_index[t] = arg max_i h[t,i] (lowest index on ties), gate[t] = p[t, expert_index[t]]
 *   position_in_expert[t] = number of earlier tokens (s < t) with the same expert
 *   dropped[t] = position_in_expert[t] >= capacity                     (Eq. 3, Fig. 3)
 *   y[t,:] = gate[t] * ReLU(x[t,:] W_in[e]) W_out[e]  if kept, +0 if dropped
 *            (the residual connection is the caller's)
 *   with noise: h is computed from x * m (Eq. 1 on the jittered input), and
 *            ReLU(.) above is followed by the dropout factor (0 or 1 / (1 - rate))
 *   SW_FFN_GEGLU: ReLU(x W_in[e]) is replaced by GELU(x W_g[e]) * (x W_l[e])
 *   ntlb_rounds > 0: for a token placed by a re-routing stage, expert_index is the expert
 *            that processes it, gate that expert's probability (which scales y),
 *            position_in_expert its slot number within the (group, expert) capacity, and
 *            dropped 0; tokens that never find a slot report the arg max, its probability
 *            and their raw rank as without re-routing.  expert_counts and aux_loss keep
 *            counting arg max decisions.
 *   aux_loss = alpha * E * sum_i f_i P_i, f_i = expert_counts[i] / T over ALL
 *            tokens (before truncation), P_i = mean_t p[t,i]            (Eqs. 4-6)
 * The workspace keeps what switch_backward needs; it must stay untouched
 * between the two calls.
 */
int switch_forward(const switch_config *cfg,
                   const void *x,               /* [T, d_model]        act_dtype            */
                   const float *W_r,            /* [d_model, E]        fp32                 */
                   const float *b_r,            /* [E] fp32 or NULL (the paper has no router bias) */
                   const void *W_in,            /* [E, d_model, d_ff]  act_dtype ([.., 2 d_ff] for SW_FFN_GEGLU) */
                   const void *W_out,           /* [E, d_ff, d_model]  act_dtype            */
                   void *y,                     /* [T, d_model]        act_dtype  (out)     */
                   int32_t *expert_index,       /* [T]   (out)                              */
                   float *gate,                 /* [T]   (out) raw top-1 probability, not masked by dropped */
                   int32_t *position_in_expert, /* [T]   (out) raw rank, defined for dropped tokens too */
                   uint8_t *dropped,            /* [T]   (out) 0 / 1                        */
                   int32_t *expert_counts,      /* [E]   (out) tokens that chose each expert, sums to T */
                   float *aux_loss,             /* [1]   (out) device scalar                */
                   float *router_logits,        /* [T, E] (out) fp32 logits, or NULL        */
                   void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Backward pass of  L = sum_t <dy[t,:], y[t,:]> + d_aux * aux_loss,
 * derived from the forward definition with f held constant (Sec. 2.2: P is
 * differentiable, f is not) and ReLU'(0) = 0.  Must follow a switch_forward
 * with the same cfg, inputs and workspace.  Dropped tokens receive only the
 * auxiliary-loss part of dx; weight-gradient blocks of experts that kept no
 * token are written as zeros.
 */
int switch_backward(const switch_config *cfg,
                    const void *dy,      /* [T, d_model] act_dtype                       */
                    float d_aux,         /* host scalar: dL/d(aux_loss)                  */
                    const void *x, const float *W_r, const float *b_r /* or NULL */,
                    const void *W_in, const void *W_out,
                    void *dx,            /* [T, d_model]       act_dtype (out)           */
                    float *dW_r,         /* [d_model, E]       fp32      (out)           */
                    float *db_r,         /* [E] fp32 (out) or NULL                       */
                    void *dW_in,         /* [E, d_model, d_ff] act_dtype (out); same shape as W_in */
                    void *dW_out,        /* [E, d_ff, d_model] act_dtype (out)           */
                    void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Forward pass without a caller workspace, for callers that cannot allocate device memory
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).
 * Same arguments, outputs and results as switch_forward, bit for bit; the workspace is a
 * fixed array of SW_STATIC_SCRATCH_BYTES of device memory inside the library (one copy per
 * GPU, held from library load until the process ends).  The call allocates and frees
 * nothing, on the device or through any library (with profiling off: switch_profile_enable
 * creates events).  A configuration whose switch_workspace_size exceeds
 * SW_STATIC_SCRATCH_BYTES is refused with SW_ERR_STATIC_LIMIT before anything else is looked
 * at.  The array keeps the previous call's contents (the forward pass reads no word of it
 * that the same call has not written, so nothing is cleared) and every call on one GPU uses
 * the same array: two such calls that overlap in time on one GPU -- different streams or
 * host threads -- race and give undefined results; calls on one stream are ordered and safe.
 * There is no backward pass on this array: switch_backward needs the workspace of a
 * switch_forward.
 */
#define SW_STATIC_SCRATCH_BYTES (32u * 1024u * 1024u)
int switch_forward_static(const switch_config *cfg, const void *x, const float *W_r,
                          const float *b_r /* or NULL */, const void *W_in, const void *W_out,
                          void *y, int32_t *expert_index, float *gate,
                          int32_t *position_in_expert, uint8_t *dropped, int32_t *expert_counts,
                          float *aux_loss, float *router_logits /* or NULL */, void *hip_stream);

/* Human-readable name of a status code.  Host; static storage. */
const char *switch_status_string(int status);

/*
 * Per-kernel timing with HIP events: for measurement only, not part of the layer's interface
 * (bench.py uses it).  While enabled, every
 * kernel the library launches is bracketed by two events recorded on the
 * call's stream.  switch_profile_collect synchronises those events and adds
 * the elapsed times to per-kernel totals; switch_profile_get reads them.
 * Host only; not thread safe; events are created on first use and kept.
 */
int switch_profile_enable(int on);         /* on != 0: start recording (clears totals) */
int switch_profile_collect(void);          /* wait for recorded events, accumulate     */
int switch_profile_count(void);            /* number of distinct kernel names seen     */
int switch_profile_get(int i, const char **name /* host, static */, double *total_ms,
                       int64_t *launches);

#ifdef __cplusplus
}
#endif
#endif /* SWITCHFFN_H */
