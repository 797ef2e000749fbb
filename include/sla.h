/*
 * libsla — Softmax Linear Attention (SLA) chunkwise-parallel forward for AMD MI355X (gfx950).
 *
 * C ABI.  Every pointer below is a DEVICE pointer unless it says "host".  The
 * caller owns every buffer; the library never frees or keeps a pointer, never
 * synchronises the device and enqueues all work on the stream it is given.
 * Functions return 0 on success and a negative sla_status on failure; on
 * failure nothing has been launched and no output has been touched.
 *
 * What one call computes, for every batch b and head h (row-vector convention,
 * state S is [dk x dv], y = q S):
 *
 *   gates (Eq. 4)          G^Q[b,t,:] = softmax over the H heads of q_head_logits[b,t,:]
 *                          G^K[b,t,:] = softmax over the H heads of k_head_logits[b,t,:]   (1 if NULL)
 *   RetNet (Sec. 5.1)      S_t = gamma_h S_{t-1} + (G^K_t k_t)^T v_t            gamma_h   = exp(log_decay[h])
 *   GLA    (Sec. 5.1)      S_t = diag(alpha_t) S_{t-1} + (G^K_t k_t)^T v_t      alpha_t,d = exp(log_decay[b,t,h,d])
 *   GDN    (Sec. 5.1)      Sb = a_t S_{t-1};  u = beta_t (G^K_t v_t - k_t Sb);  S_t = Sb + k_t^T u
 *                                                                               a_t = exp(log_decay[b,t,h])
 *   read-out (Eq. 5-6)     out[b,t,h,:] = G^Q_t (q_t S_t)      -- the state after token t
 *   final_state[b,h]       = S_T
 *
 * It is evaluated in the chunkwise-parallel form of Sec. 3.2 ("Chunkwise
 * Parallel Training"): matrix products inside blocks of tokens, the state
 * carried between blocks in fp32; the result does not depend on the blocking
 * beyond rounding.  q and k are taken as given: the feature map, any 1/sqrt(d)
 * scaling or L2 normalisation, and the projections that produce the gate
 * logits (Eq. 4) and consume the output (Eq. 7) are the caller's.
 *
 * Domain: every log-decay must be <= 0; for GLA each must also be >= -5
 * (the blocked evaluation divides keys by the decay accumulated inside a block of
 * 16 tokens; below e^-5 per token that quotient leaves the fp32 range and results
 * may be inf/NaN).  RetNet and GDN take any decay <= 0.  A GLA block whose
 * accumulated decay falls below e^-80 is reported: the kernels set
 * SLA_DEVICE_DECAY_RANGE in the device status word (sla_device_status).
 * NaN or infinite inputs propagate to the outputs; they are not trapped.
 */
#ifndef SLA_H_
#define SLA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Which recurrence of Sec. 5.1 ("Instantiations on Linear Baselines") to run. */
typedef enum { SLA_RETNET = 0, SLA_GLA = 1, SLA_GDN = 2 } sla_variant;

/* Element type of q, k, v, out (and of the GLA log_decay).  Accumulation and the state are fp32. */
typedef enum { SLA_F32 = 0, SLA_BF16 = 1 } sla_dtype;

typedef enum {
    SLA_OK = 0,
    SLA_ERR_NULL = -1,        /* a required pointer is NULL, or a pointer that must be NULL is not */
    SLA_ERR_SHAPE = -2,       /* a size is negative or out of range */
    SLA_ERR_UNSUPPORTED = -3, /* variant / dtype / head dimension not built */
    SLA_ERR_ALIGN = -4,       /* a pointer is not 16-byte aligned */
    SLA_ERR_HIP = -5,         /* the HIP runtime refused the launch (no device, bad stream, ...) */
    SLA_ERR_WORKSPACE = -6,   /* segments > 1 asked for, but no workspace or too small a one was given */
    SLA_ERR_SCRATCH = -7      /* sla_forward_static: the schedule needs more than SLA_STATIC_SCRATCH_BYTES */
} sla_status;

/* sla_params.flags.  SLA_FLAG_HEAD_MAJOR: q, k, v, out and the GLA log_decay are laid out [B,H,T,d] instead of
 * [B,T,H,d], so that every (batch, head) pair streams one contiguous region of memory (measurably kinder to the
 * DRAM than 256-byte pieces 4 KB apart).  For sla_backward the same holds for d_out, dq, dk, dv and dlog_decay.
 * Logits and their gradients, beta, the delta rule's decay and the states keep their layouts. */
#define SLA_FLAG_HEAD_MAJOR 1

/* Problem description (host memory, read during the call only). */
typedef struct {
    int32_t variant; /* sla_variant */
    int32_t dtype;   /* sla_dtype */
    int32_t B;       /* batch size            >= 0 */
    int32_t T;       /* tokens per sequence   >= 0 */
    int32_t H;       /* heads                 1..64 */
    int32_t dk;      /* key/query head width  32, 64 or 128 (32: the backward passes run it zero-padded to 64, single
                        pass only, with the padded copies in their workspace) */
    int32_t dv;      /* value head width      64, 128 or 256 */
    int32_t dv_split; /* 0 = let the library choose; else value columns per workgroup: 16, 32 or 64 (<= dv).
                        A scheduling knob only: results are bit-identical for every width
                        (each output column is computed by exactly one workgroup in a fixed order). */
    int32_t flags;   /* 0, or SLA_FLAG_HEAD_MAJOR for sla_forward / sla_forward_ws / sla_backward (every other entry
                        point: 0) */
    int32_t segments; /* schedule for shapes with few (batch, head) pairs, RetNet and GLA only: T is cut into
                         this many segments that run in parallel (a pre-pass computes each segment's end state
                         from a zero entry state, a small kernel chains them through the segments' decays, the
                         main pass starts every segment from its entry state).  0 = the library chooses when a
                         workspace is given (1 when there are enough rows to fill the device); 1 = one fused
                         pass.  The result is the same up to fp32 rounding of the chained states.  sla_backward
                         cuts only on request (>= 2), see there. */
} sla_params;

/*
 * SLA forward, Eq. 3-6 with the Sec. 5.1 recurrences, chunkwise-parallel (Sec. 3.2).
 *
 *   q, k            [B,T,H,dk]  dtype   feature-mapped queries / keys
 *   v               [B,T,H,dv]  dtype
 *   q_head_logits   [B,T,H]     fp32    read-gate scores  (Q W_GQ in Eq. 4); required
 *   k_head_logits   [B,T,H]     fp32    write-gate scores (K W_GK in Eq. 4); NULL means G^K = 1
 *   log_decay       RetNet: fp32 [H];  GLA: dtype [B,T,H,dk];  GDN: fp32 [B,T,H]
 *   beta            GDN: fp32 [B,T,H] in [0,1]; must be NULL for RetNet and GLA
 *   initial_state   [B,H,dk,dv] fp32, or NULL for a zero state
 *   out             [B,T,H,dv]  dtype   written
 *   final_state     [B,H,dk,dv] fp32    written; NULL to skip.  May alias initial_state.
 *   stream          a hipStream_t passed as void* (NULL = the default stream)
 *
 * sla_forward always runs one fused pass (p->segments must be 0 or 1); see sla_forward_ws.
 *
 * All tensors are dense and row-major in the index order shown; pointers must
 * be 16-byte aligned.  B == 0 is a no-op.  T == 0 copies initial_state (or
 * zeros) to final_state.  Asynchronous: returns after enqueueing.
 */
int sla_forward(const sla_params* p, const void* q, const void* k, const void* v,
                const float* q_head_logits, const float* k_head_logits,
                const void* log_decay, const float* beta, const float* initial_state,
                void* out, float* final_state, void* stream);

/*
 * sla_forward with a workspace (device memory, 16-byte aligned, owned by the caller, contents undefined on
 * return), which lets the library use the segment-parallel schedule described at sla_params.segments: the
 * sequential state carry between chunks of Sec. 3.2 (Chunkwise Parallel Training) becomes a two-level scan.
 * workspace may be NULL (then this is sla_forward).  With p->segments == 0 a workspace that is too small makes
 * the call fall back to one fused pass; with p->segments > 1 it is SLA_ERR_WORKSPACE.
 */
int sla_forward_ws(const sla_params* p, const void* q, const void* k, const void* v,
                   const float* q_head_logits, const float* k_head_logits,
                   const void* log_decay, const float* beta, const float* initial_state,
                   void* out, float* final_state, void* workspace, size_t workspace_bytes, void* stream);

/*
 * sla_forward_ws for callers that cannot allocate device memory and have no workspace to hand in: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and results as sla_forward;
 * the schedule is the one sla_forward_ws would choose with a large enough workspace (p->segments as there), and the
 * workspace is a buffer of SLA_STATIC_SCRATCH_BYTES that is part of the library's device image (every GPU the
 * library runs on holds one copy until the process ends).  The call allocates and frees nothing.
 *
 * Limit: a shape whose segment schedule needs more than SLA_STATIC_SCRATCH_BYTES is rejected with SLA_ERR_SCRATCH
 * and nothing is launched (the five benchmark shapes and the paper-shape workloads need at most 8.8 MB; shapes
 * that run as one fused pass, the delta rule among them, need none).  Use sla_forward_ws for larger ones.
 * All calls on one GPU share that GPU's buffer: calls that may overlap in time on one GPU (different streams,
 * different host threads) race on it and must be serialised by the caller.  Nothing in the buffer has to survive
 * between calls and nothing in it has to start at zero; its contents after a call are undefined.
 *
 * sla_init resolves the buffer's device address for the current device ahead of time (optional: the first
 * sla_forward_static on a device does the same); call it once per device before capturing a graph, so that the
 * captured call itself only launches kernels.  Returns SLA_OK or SLA_ERR_HIP.
 */
#define SLA_STATIC_SCRATCH_BYTES (16u << 20)
int sla_init(void);
size_t sla_static_scratch_bytes(void);
int sla_forward_static(const sla_params* p, const void* q, const void* k, const void* v,
                       const float* q_head_logits, const float* k_head_logits,
                       const void* log_decay, const float* beta, const float* initial_state,
                       void* out, float* final_state, void* stream);

/*
 * One recurrent decode step: Eq. 5-6 with the Sec. 5.1 recurrences for a single token per (batch, head), the
 * constant-memory inference form (Sec. 3.2, Recurrent Implementation; Appendix A, Derivation of Recurrent
 * Implementation; decode latency is what Sec. 5.7, Training Efficiency, reports for it).  Exactly
 * sla_forward for T = 1 with initial_state = final_state = state, as one streaming read-modify-write of the
 * state.  p->T must be 1; dv_split and segments are ignored.
 *
 *   q, k            [B,H,dk]    dtype
 *   v               [B,H,dv]    dtype
 *   q_head_logits   [B,H]       fp32; k_head_logits [B,H] fp32 or NULL (G^K = 1)
 *   log_decay       RetNet: fp32 [H];  GLA: dtype [B,H,dk];  GDN: fp32 [B,H]
 *   beta            GDN: fp32 [B,H]; NULL otherwise
 *   state           [B,H,dk,dv] fp32    read and overwritten with the state after the token; required
 *   out             [B,H,dv]    dtype   written
 */
int sla_decode_step(const sla_params* p, const void* q, const void* k, const void* v,
                    const float* q_head_logits, const float* k_head_logits,
                    const void* log_decay, const float* beta, float* state, void* out, void* stream);

/*
 * The decode step with the gate projection of Sec. 3.2 fused in: instead of logits it takes the two gate matrices
 * (as sla_gate_logits does) and forms q_head_logits[b,h'] = q[b,h',:] . W_GQ[:,h'] (and the same for k) for every
 * head h' of the token inside the kernel, then the head softmax of Eq. 4 and the step of sla_decode_step.  A
 * decode step sees the whole token anyway, so the projection costs 2 H dk multiply-adds per workgroup and saves a
 * launch per generated token.  The logits are formed in fp32 from the tensors as given; the result equals
 * sla_gate_logits followed by sla_decode_step up to the order of the fp32 sums.
 *
 *   w_gq   [H,dk] fp32   device, read only: row h is column h of the paper's matrix; required
 *   w_gk   [H,dk] fp32   or NULL (G^K = 1)
 * Everything else as sla_decode_step.
 */
int sla_decode_step_fused(const sla_params* p, const void* q, const void* k, const void* v,
                          const float* w_gq, const float* w_gk,
                          const void* log_decay, const float* beta, float* state, void* out, void* stream);

/*
 * Backward pass of sla_forward for the RetNet and GLA recurrences (Sec. 5.1) with the gates of Eq. 4-6: the
 * gradients that training through the chunkwise form of Sec. 3.2 (Chunkwise Parallel Training) needs.  With the
 * scalar objective L = sum(out * d_out) + sum(final_state * d_final_state) it writes dL/d(input) for every
 * differentiable input of the forward call made with the same p, q, k, v, logits, log_decay and initial_state.
 * bf16 tensors run in block form on the matrix cores; fp32 tensors (p->dtype == SLA_F32) run token by token in fp32
 * vector arithmetic (gradients to fp32 rounding, any log_decay <= 0, single pass only: p->segments >= 2 is
 * SLA_ERR_UNSUPPORTED).  The delta rule has its own entry point, sla_backward_gdn.
 * p->dv_split is ignored.  p->segments >= 2 asks for the segment-parallel schedule (for batches with few sequences,
 * as in sla_forward_ws): every batch row is cut into that many segments (of a multiple of 64 tokens, at least 256)
 * which run in parallel; the entry state and the end cotangent of every segment come from two pre-passes.  It needs
 * the [B,T,H,d] layout (p->flags == 0) and a larger workspace (sla_backward_workspace_bytes accounts for it); 0 and 1
 * run the single pass.
 *
 *   q, k, v, q_head_logits, k_head_logits, log_decay, initial_state   as for sla_forward (device, read only)
 *   d_out            [B,T,H,dv]  dtype   cotangent of out; required
 *   d_final_state    [B,H,dk,dv] fp32    cotangent of final_state, or NULL (zero)
 *   dq, dk           [B,T,H,dk]  dtype   written
 *   dv               [B,T,H,dv]  dtype   written
 *   dq_head_logits   [B,T,H]     fp32    written (through the head softmax)
 *   dk_head_logits   [B,T,H]     fp32    written; required when k_head_logits is given, NULL otherwise
 *   dlog_decay       GLA: [B,T,H,dk] dtype, written, required;  RetNet: must be NULL (the decay is a constant)
 *   d_initial_state  [B,H,dk,dv] fp32    written, or NULL (not wanted)
 *   workspace        device memory of at least sla_backward_workspace_bytes(p) bytes, 16-byte aligned; holds
 *                    the gates, partial gate gradients and (GLA, bf16) block sums of q * dq and the state entering
 *                    every 512th token of a sequence (dlog_decay is re-derived from rowsum(dS * S) there, so its
 *                    error does not grow with the sequence length).  Contents on entry are ignored; calls that
 *                    share a workspace must not overlap.
 * No output may overlap an input or another output.  Everything is enqueued on `stream`; nothing is allocated,
 * freed or synchronised.  Returns a status code; on error nothing is launched.
 */
int sla_backward(const sla_params* p, const void* q, const void* k, const void* v,
                 const float* q_head_logits, const float* k_head_logits, const void* log_decay,
                 const float* initial_state, const void* d_out, const float* d_final_state,
                 void* dq, void* dk, void* dv, float* dq_head_logits, float* dk_head_logits,
                 void* dlog_decay, float* d_initial_state,
                 void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of workspace sla_backward needs for *p (0 when *p is not a shape it supports). */
size_t sla_backward_workspace_bytes(const sla_params* p);

/*
 * Backward pass of sla_forward for the gated delta rule (Softmax-GatedDeltaNet, Sec. 5.1, with the gates of
 * Eq. 4-6): p->variant must be SLA_GDN and p->flags 0 (else SLA_ERR_UNSUPPORTED); bf16 or fp32 tensors.  Same objective
 * and conventions as sla_backward; the step differentiated is
 *     Sb = exp(log_decay_t) S_{t-1},  u = beta_t (G^K_t v_t - k_t Sb),  S_t = Sb + k_t^T u,  out_t = G^Q_t q_t S_t.
 *
 *   q, k, v, q_head_logits, k_head_logits, initial_state, d_out, d_final_state,
 *   dq, dk, dv, dq_head_logits, dk_head_logits, d_initial_state      as for sla_backward
 *   log_decay, beta  [B,T,H] fp32   as for sla_forward; required.  fp32 tensors: log_decay >= -20 per token (those
 *                                   sweeps keep their state divided by the decay product of up to four tokens)
 *   dlog_decay       [B,T,H] fp32   written; required
 *   dbeta            [B,T,H] fp32   written; required
 *   workspace        device memory of at least sla_backward_gdn_workspace_bytes(p) bytes, 16-byte aligned (gates,
 *                    partial sums, and what passes the delta rule's feedback terms between the four sweeps: three
 *                    tensors the size of v, v and k, in fp32 for fp32 tensors; in bf16, with one 32 x 32 matrix and
 *                    256 scalars per 32-token block and head and the state cotangent at every 512th token of a
 *                    sequence, for bf16 tensors).  Contents on entry are ignored; calls that share a workspace must
 *                    not overlap.
 * bf16 tensors run in block form on the matrix cores (32-token blocks, fp32 accumulation, every decay factor <= 1;
 * dlog_decay is re-derived exactly every 512 tokens, so its error does not grow with the sequence length); fp32
 * tensors run token by token in fp32 vector arithmetic.
 * Everything is enqueued on `stream`; nothing is allocated, freed or synchronised.  Returns a status code; on error
 * nothing is launched.
 */
int sla_backward_gdn(const sla_params* p, const void* q, const void* k, const void* v,
                     const float* q_head_logits, const float* k_head_logits, const float* log_decay,
                     const float* beta, const float* initial_state, const void* d_out,
                     const float* d_final_state, void* dq, void* dk, void* dv, float* dq_head_logits,
                     float* dk_head_logits, float* dlog_decay, float* dbeta, float* d_initial_state,
                     void* workspace, size_t workspace_bytes, void* stream);
size_t sla_backward_gdn_workspace_bytes(const sla_params* p);

/*
 * The same on a packed batch of sequences of different lengths, with the conventions of sla_forward_varlen /
 * sla_backward_varlen: p->T is the total number of tokens, p->B the number of sequences, cu_seqlens [B+1] int32 in
 * DEVICE memory (clamped into [0, p->T] by the kernels), one state per sequence; log_decay, beta and their gradients
 * are [T,H].  Needs sla_backward_gdn_varlen_workspace_bytes(p) bytes of workspace.
 */
int sla_backward_gdn_varlen(const sla_params* p, const void* q, const void* k, const void* v,
                            const float* q_head_logits, const float* k_head_logits, const float* log_decay,
                            const float* beta, const int32_t* cu_seqlens, const float* initial_state,
                            const void* d_out, const float* d_final_state, void* dq, void* dk, void* dv,
                            float* dq_head_logits, float* dk_head_logits, float* dlog_decay, float* dbeta,
                            float* d_initial_state, void* workspace, size_t workspace_bytes, void* stream);
size_t sla_backward_gdn_varlen_workspace_bytes(const sla_params* p);

/*
 * Gate logits: the scores Eq. 4 takes the head softmax of, from the (feature-mapped) queries and keys and the
 * two gate matrices W_GQ, W_GK in R^{d x H} of Sec. 3.2, with d the head width (the reading under which the two
 * matrices add the 0.05 M parameters that the "Parameter Efficiency" paragraph counts):
 *     q_head_logits[b,t,h] = q[b,t,h,:] . W_GQ[:,h]        k_head_logits[b,t,h] = k[b,t,h,:] . W_GK[:,h]
 * One streaming pass over q and k; the result is what sla_forward / sla_backward take as logits.
 *
 *   q, k             [B,T,H,dk]  dtype   device, read only; k may be NULL (then w_gk and k_head_logits must be too)
 *   w_gq, w_gk       [H,dk]      fp32    device, read only: row h is column h of the paper's matrix
 *   q_head_logits    [B,T,H]     fp32    written
 *   k_head_logits    [B,T,H]     fp32    written, or NULL with k
 * Uses p->dtype, B, T, H, dk (dv, variant, dv_split, segments are validated as for sla_forward and otherwise
 * ignored).  Enqueued on `stream`; nothing is allocated or synchronised.  Returns a status code.
 */
int sla_gate_logits(const sla_params* p, const void* q, const void* k, const float* w_gq, const float* w_gk,
                    float* q_head_logits, float* k_head_logits, void* stream);

/*
 * Packed variable-length batches: p->B sequences laid end to end along the token axis, as language-model
 * training on documents of mixed length feeds the mixer (the training runs of Sec. 5.2 use 4K-token contexts;
 * Sec. 5.3's retrieval lengths range from 1K to 8K and beyond).  p->T is the TOTAL number of tokens, the tensors
 * have the layouts of sla_forward with a single batch row of p->T tokens, and sequence b covers tokens
 * cu_seqlens[b] .. cu_seqlens[b+1]-1.  Every sequence has its own state: the recurrence of Eq. 5 restarts at each
 * boundary from initial_state[b] (zero if NULL) and leaves final_state[b].
 *
 *   cu_seqlens       [B+1] int32, DEVICE memory, read by the kernels: non-decreasing, cu_seqlens[0] >= 0,
 *                    cu_seqlens[B] <= p->T (tokens outside every sequence are neither read nor written; offsets
 *                    are clamped into [0, p->T], so no content of this array makes the kernels leave the tensors)
 *   initial_state, final_state, d_final_state, d_initial_state   [B,H,dk,dv] fp32, one per sequence
 *   everything else as for sla_forward / sla_backward with batch size 1 and T = p->T
 * One fused pass per sequence and slice (p->segments > 1 is SLA_ERR_UNSUPPORTED); empty sequences pass their
 * state through.  sla_backward_varlen needs sla_backward_varlen_workspace_bytes(p) bytes of workspace.
 */
int sla_forward_varlen(const sla_params* p, const void* q, const void* k, const void* v,
                       const float* q_head_logits, const float* k_head_logits,
                       const void* log_decay, const float* beta, const int32_t* cu_seqlens,
                       const float* initial_state, void* out, float* final_state, void* stream);
int sla_backward_varlen(const sla_params* p, const void* q, const void* k, const void* v,
                        const float* q_head_logits, const float* k_head_logits, const void* log_decay,
                        const int32_t* cu_seqlens, const float* initial_state, const void* d_out,
                        const float* d_final_state, void* dq, void* dk, void* dv, float* dq_head_logits,
                        float* dk_head_logits, void* dlog_decay, float* d_initial_state,
                        void* workspace, size_t workspace_bytes, void* stream);
size_t sla_backward_varlen_workspace_bytes(const sla_params* p);

/*
 * Short causal convolution along the tokens followed by SiLU, per channel: the feature map that the Gated DeltaNet
 * blocks of Sec. 5.1 ("Model Configuration": short-convolution module and SiLU) apply in front of q and k (and v),
 *     y[b,t,c] = silu( sum_{i < taps} w[c,i] * x[b, t - (taps-1) + i, c] ),   x = 0 before the sequence.
 * One streaming pass; call it once per tensor.  Rectangular batches only (a packed batch would need the window to
 * stop at sequence boundaries).
 *
 *   x, y    [B,T,channels]  dtype   device; y written; must not overlap
 *   w       [channels,taps] fp32    device; tap taps-1 multiplies the current token
 *   channels a multiple of 8, 8 .. 65536;  taps 1 .. 4;  dtype SLA_F32 or SLA_BF16;  B, T >= 0
 */
int sla_short_conv_silu(int dtype, int B, int T, int channels, int taps, const void* x, const float* w, void* y,
                        void* stream);

/*
 * The same feature map with an optional L2 normalisation of every head's vector behind it (the benchmark's delta-rule
 * workload feeds L2-normalised queries and keys; the paper's Sec. 5.1 names only the convolution and SiLU, so this
 * is an option): with head_width > 0 every group of head_width adjacent channels of a token is divided by
 * sqrt(sum of its squares + eps).  head_width 0 (no normalisation), 32, 64 or 128; with head_width > 0 channels must
 * be a multiple of 128 and eps >= 0.  Otherwise as sla_short_conv_silu.
 */
int sla_short_conv_silu_l2(int dtype, int B, int T, int channels, int taps, int head_width, float eps, const void* x,
                           const float* w, void* y, void* stream);

/*
 * Backward of sla_short_conv_silu_l2 (of sla_short_conv_silu with head_width = 0): for the cotangent dy of y,
 *     dx [B,T,channels] dtype  written (must not overlap x, dy)
 *     dw [channels,taps] fp32  written (sum over all tokens, taken in a fixed order: bitwise reproducible)
 * The convolution is recomputed from x and w, nothing is kept from the forward call.  workspace: device memory of
 * sla_short_conv_silu_l2_backward_workspace_bytes(B, T, channels, taps) bytes (partial sums of dw), 16-byte aligned.
 * B == 0 or T == 0 is a no-op that leaves dw untouched.
 */
int sla_short_conv_silu_l2_backward(int dtype, int B, int T, int channels, int taps, int head_width, float eps,
                                    const void* x, const float* w, const void* dy, void* dx, float* dw,
                                    void* workspace, size_t workspace_bytes, void* stream);
size_t sla_short_conv_silu_l2_backward_workspace_bytes(int B, int T, int channels, int taps);

/*
 * Backward of one gate projection of sla_gate_logits (Eq. 4's scores, logits[b,t,h] = x[b,t,h,:] . W[:,h]); call it
 * once for the queries (x = q, w = w_gq, the mixer's dq_head_logits and dq) and once for the keys:
 *     x              [B,T,H,dk] dtype   the projected tensor (device, read only)
 *     w              [H,dk] fp32        as for sla_gate_logits
 *     d_head_logits  [B,T,H] fp32       cotangent of the logits (what sla_backward / sla_backward_gdn return)
 *     dx             [B,T,H,dk] dtype   READ AND UPDATED IN PLACE: dx[b,t,h,:] += d_head_logits[b,t,h] w[h,:]
 *                                       (pass the dq / dk that the mixer's backward has written)
 *     dw             [H,dk] fp32        written: sum over b, t of d_head_logits[b,t,h] x[b,t,h,:] (fixed order)
 *     workspace      sla_gate_logits_backward_workspace_bytes(p) bytes of device memory, 16-byte aligned
 * Uses p->dtype, B, T, H, dk; p->flags must be 0.
 */
int sla_gate_logits_backward(const sla_params* p, const void* x, const float* w, const float* d_head_logits, void* dx,
                             float* dw, void* workspace, size_t workspace_bytes, void* stream);
size_t sla_gate_logits_backward_workspace_bytes(const sla_params* p);

/* Bytes of workspace sla_forward_ws wants for *p on a device with that many compute units (0: none needed). */
size_t sla_workspace_bytes(const sla_params* p, int compute_units);

/* Number of segments the library would choose for *p given a workspace (>= 1); <0 on error. */
int sla_segments(const sla_params* p, int compute_units);

/*
 * Number of segments to put into p->segments for sla_backward on a device with that many compute units (>= 1; 1 when
 * the single pass already gives every compute unit a workgroup, or for the delta rule); <0 on error.  The narrowest
 * of the three sweeps runs B * H * min(dk, dv) / 64 workgroups per segment.  sla_backward itself never chooses:
 * its workspace size must not depend on the device.
 */
int sla_backward_segments(const sla_params* p, int compute_units);

/*
 * Validates the same arguments as sla_forward (host-side checks only, touches no
 * device and launches nothing).  Returns what sla_forward would return before
 * its first HIP call.
 */
int sla_check_args(const sla_params* p, const void* q, const void* k, const void* v,
                   const float* q_head_logits, const float* k_head_logits,
                   const void* log_decay, const float* beta, const float* initial_state,
                   const void* out, const float* final_state);

/* Value columns per workgroup the library would choose for *p (the dv_split it resolves 0 to); <0 on error.
 * p->segments <= 1: the choice for one fused pass; > 1: the choice for that many segments. */
int sla_default_dv_split(const sla_params* p, int compute_units);

/* Name of the device kernel that sla_forward launches for *p (static string, host memory); NULL on error.
 * Lets a profiler summary be matched to a call. */
const char* sla_kernel_name(const sla_params* p);

/*
 * Device status word: things a kernel noticed that no return code can carry, because every entry point returns
 * before its kernels run.  One sticky word per GPU, OR-ed into by the kernels of every call on that GPU:
 *   SLA_DEVICE_WAIT_EXPIRED  a producer/consumer hand-over inside a workgroup gave up waiting (each wait is bounded
 *                            so that no wave can hang).  It cannot happen in a correct run; if it is ever set, the
 *                            outputs of the calls since the last reset are invalid.
 *   SLA_DEVICE_DECAY_RANGE   a GLA forward saw a 16-token block whose accumulated decay is below e^-80 (a log-decay
 *                            under the documented -5 per token, or a NaN): results may hold inf/NaN.
 * sla_device_status copies the word of the current device to *status (host memory) after waiting for `stream`, and
 * clears it when `reset` is non-zero.  It synchronises the stream: not for use under graph capture.  Returns SLA_OK,
 * SLA_ERR_NULL or SLA_ERR_HIP.
 */
#define SLA_DEVICE_WAIT_EXPIRED 1u
#define SLA_DEVICE_DECAY_RANGE 2u
int sla_device_status(uint32_t* status, int reset, void* stream);

/* Human-readable text for a status code (static string, host memory). */
const char* sla_status_string(int status);

/* Library version: major*10000 + minor*100 + patch. */
int sla_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SLA_H_ */
