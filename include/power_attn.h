/*
 * power_attn.h -- C ABI of the MI355X (gfx950) chunked causal power-attention library.
 *
 * The layer (arXiv 2507.04239, Sec. 4 Eq. (7), with the sum-of-scores normalisation of
 * Sec. 2 "Normalization" / App. E.4), per batch b and head h, for i = 0..T-1:
 *
 *     s_ij = scale * (q_i . k_j)            j <= i   (causal, diagonal included)
 *     N_i  = sum_{j<=i} s_ij^p v_j          Z_i = sum_{j<=i} s_ij^p
 *     O_i  = N_i / Z_i  (normalize != 0)    or    O_i = N_i  (normalize == 0)
 *
 * It is evaluated in the chunked form of Sec. 2 "Chunked form" / App. A and E: the state
 * S_n = sum_{j < n*chunk} phi(k_j) [v_j, 1]^T over a (tiled) symmetric-power embedding phi
 * (Lemma 4.2, Sec. 4.1.1) is accumulated chunk by chunk (update-state, App. E.2, plus the
 * un-gated cumulative sum of App. E.3), read out with phi(q_i) (query-state, App. E.4), and
 * combined with the attention form inside each chunk (App. E.1).  phi(q), phi(k) exist only
 * in registers / LDS.  The backward pass (not in the paper) differentiates exactly the
 * function above.
 *
 * All pointers named Q, K, V, O, Z, dO, dQ, dK, dV and `workspace` are DEVICE pointers
 * (HIP global memory on the current device); `const pa_problem*` and the profiling
 * arguments are HOST pointers.  Tensors are dense row-major [B, H, T, d] (Q, K, dQ, dK),
 * [B, H, T, v] (V, O, dO, dV) in `dtype`, and [B, H, T] float32 (Z, log_g, dlog_g).  Every
 * tensor pointer must be 16-byte aligned (they are accessed with 16-byte vector loads and
 * stores) and every workspace 256-byte aligned; a misaligned pointer is PA_ERR_INVALID_ARG
 * (PA_ERR_WORKSPACE for a workspace) and nothing is launched.  The caller owns every buffer;
 * the library allocates no device memory, keeps no per-call state and enqueues work on
 * `hip_stream` (a hipStream_t passed as void*, NULL = the default stream); it does not
 * synchronise the host.  One exception to "only on hip_stream": the bf16 MFMA backward pass
 * runs independent kernels side by side on one more stream (non-blocking, default priority),
 * forked from and joined back into hip_stream with events, so that for the caller the call
 * is ordered on hip_stream like any other.
 * Host threads: what the library keeps between calls is kept per host thread - that side
 * stream and its events (created on the thread's first such call, destroyed by
 * power_attn_release_thread), the text of the last HIP error, and the profiling switch with
 * its records - so calls may be issued concurrently from several host threads, each on a
 * stream and buffers of its own.  The exception is power_attn_fwd_static, whose scratch is
 * one array per GPU.  Outputs are overwritten, never accumulated into.
 * No function throws; all errors are return codes and nothing is launched when
 * validation fails.
 */
#ifndef POWER_ATTN_H
#define POWER_ATTN_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PA_OK = 0,
    PA_ERR_INVALID_ARG = 1,   /* null pointer, non-positive size, odd p with normalize, ... */
    PA_ERR_UNSUPPORTED = 2,   /* a valid problem this build has no kernel for (see pa_problem) */
    PA_ERR_WORKSPACE   = 3,   /* workspace is NULL or smaller than power_attn_workspace_bytes() */
    PA_ERR_HIP         = 4    /* a HIP runtime call or kernel launch failed */
} pa_status;

typedef enum { PA_DTYPE_F32 = 0, PA_DTYPE_BF16 = 1 } pa_dtype;

/* Which kernel family evaluates the problem.  AUTO picks MFMA when it applies. */
typedef enum {
    PA_IMPL_AUTO    = 0,
    PA_IMPL_GENERIC = 1,  /* float32 arithmetic on the vector ALUs; any 1 <= p <= 4, d, v <= 128; both dtypes */
    PA_IMPL_MFMA    = 2,  /* bf16 MFMA with float32 accumulation; bf16 only.  Chunked form: p = 2, d = v = 64,
                             chunk a multiple of 128.  Attention form (chunk == T; any T, or with
                             gates T a multiple of 128, of 256 at d = 32): p in {2, 3, 4}, d = v in {32, 64, 128}.  See power_attn_supported() */
    PA_IMPL_RESIDENT = 3, /* the chunked bf16 MFMA kernels that keep the chunk states in registers while they walk the
                             sequence (no chunk state is written to memory): p = 2, d = v in {64, 128}, chunk a multiple
                             of 128, not gated */
    PA_IMPL_TILED = 4     /* the chunked bf16 MFMA kernels with the degree and the tile width of the embedding
                             (Sec. 4.1.1) as parameters, chunk states in memory: d = v = 32 with (p, d_tile) in
                             {(2,4), (2,8), (2,16), (3,4), (4,2), (4,4)}, d = v = 64 with {(2,4), (2,8), (2,16), (3,4)},
                             d = v = 128 with (2,8); chunk a multiple of 128 that divides T, at least two chunks, not
                             gated.  What AUTO runs for the chunked form of p = 3 and p = 4, of d = 32, and of p = 2
                             at d = 128 */
} pa_impl;

typedef struct {
    int   B, H, T;      /* batch, heads, sequence length */
    int   d;            /* query / key head size */
    int   v;            /* value head size */
    int   p;            /* degree of the power (Sec. 4 Eq. (7)); even when normalize != 0 */
    int   chunk;        /* chunk size c of the chunked form.  chunk == T is the attention form (one chunk).
                           0: the library chooses between the two forms and the chunk size (see
                           power_attn_resolved_chunk).  A chunk that does not divide T (a ragged last
                           chunk) is taken by the chunked bf16 MFMA kernels only, which then run the
                           sequence padded with zero rows inside the workspace; elsewhere it is
                           PA_ERR_UNSUPPORTED */
    int   normalize;    /* 1: divide by the sum of the scores; 0: leave un-normalised */
    float scale;        /* multiplies q.k before the power ("softmax scaling", App. E.1 step 2) */
    int   dtype;        /* pa_dtype of Q, K, V, O, dO, dQ, dK, dV; accumulation is always float32 */
    int   impl;         /* pa_impl */
    int   keep_state;   /* 0: power_attn_bwd rebuilds the chunk states itself (nothing but O and Z is
                           saved).  1: power_attn_fwd also leaves the chunk states in `workspace` in
                           the form the backward pass reads, and power_attn_bwd, given the SAME
                           workspace, untouched since, and the same problem and inputs, uses them
                           instead of rebuilding.  Both calls then need
                           power_attn_workspace_bytes(prob, 1) bytes.  A kernel family may ignore
                           the hint and rebuild. */
    int   gated;        /* 0: the layer above (power_attn_fwd / power_attn_bwd).  1: gated
                           (power_attn_fwd_gated / power_attn_bwd_gated): with one log-gate
                           log g_t <= 0 per batch, head and timestep (Sec. 2 "Gating"; the decay of
                           App. E.2 / E.3 at timestep granularity) and b_i = sum_{t<=i} log g_t, the
                           pair (i, j) is weighted by the gates of the steps j+1 .. i:
                               a_ij = s_ij^p exp(b_i - b_j),
                           N_i = sum_j a_ij v_j, Z_i = sum_j a_ij. */
    int   d_tile;       /* tile width of the tiled symmetric-power embedding (Sec. 4.1.1).  0: the kernel family's
                           own (8 for p = 2, 4 for p = 3, 2 for p = 4).  A value > 0 asks for the PA_IMPL_TILED kernels
                           with that width (PA_ERR_UNSUPPORTED if they do not take the problem); the result does
                           not depend on it beyond rounding. */
} pa_problem;

/* Bytes of device scratch the calls below need for `prob` (0 on an invalid problem).
 * for_backward = 0: power_attn_fwd; 1: power_attn_bwd. */
size_t power_attn_workspace_bytes(const pa_problem* prob, int for_backward);

/* PA_OK if `prob` is valid and a kernel family exists under prob->impl for its forward
 * (for_backward = 0) or backward (1) pass. */
pa_status power_attn_supported(const pa_problem* prob, int for_backward);

/* Forward pass.  Writes O [B,H,T,v] and Z [B,H,T] (Z_i = the row's sum of scores, saved for
 * the backward pass; Z may be NULL when it is not wanted).  A row with Z_i == 0 gets O_i = 0
 * when normalize != 0 (the paper is silent on it). */
pa_status power_attn_fwd(const pa_problem* prob,
                         const void* Q, const void* K, const void* V,
                         void* O, float* Z,
                         void* workspace, size_t workspace_bytes, void* hip_stream);

/* power_attn_fwd for callers that cannot allocate device memory and have no workspace to hand over
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same
 * kernels as power_attn_fwd, with the workspace taken from a device array that is part of the
 * library itself (PA_STATIC_SCRATCH_BYTES, one copy per GPU, held until the process ends).  The call
 * allocates nothing.  A problem whose power_attn_workspace_bytes(prob, 0) exceeds
 * power_attn_static_scratch_bytes() is refused with PA_ERR_WORKSPACE and nothing is launched
 * (prob->keep_state is honoured only in the sense that the states stay in that array).  All calls
 * on one GPU share the array: calls that overlap on one GPU (different streams or host threads)
 * race; calls on one stream are ordered and safe.  Everything else as power_attn_fwd. */
#define PA_STATIC_SCRATCH_BYTES (16u << 20)
size_t power_attn_static_scratch_bytes(void);
pa_status power_attn_fwd_static(const pa_problem* prob,
                                const void* Q, const void* K, const void* V,
                                void* O, float* Z, void* hip_stream);

/* Backward pass: given dO = dL/dO and the forward outputs O, Z of the same problem and
 * inputs, writes dQ, dK, dV.  (O and Z are read only when normalize != 0.)  Rows with
 * Z_i == 0 pass no gradient. */
pa_status power_attn_bwd(const pa_problem* prob,
                         const void* Q, const void* K, const void* V,
                         const void* O, const float* Z, const void* dO,
                         void* dQ, void* dK, void* dV,
                         void* workspace, size_t workspace_bytes, void* hip_stream);

/* Gated layer (prob->gated == 1).  log_g: DEVICE float32 [B,H,T], values <= 0 (a positive
 * value is a growth factor: accepted, but the chunked evaluation may then overflow).  The
 * backward pass also writes dlog_g [B,H,T] float32 = dL/dlog g_t (dlog_g of the first timestep
 * is 0: no pair straddles it).  Everything else as in the un-gated calls; the un-gated calls
 * refuse a gated problem and vice versa (PA_ERR_INVALID_ARG). */
pa_status power_attn_fwd_gated(const pa_problem* prob,
                               const void* Q, const void* K, const void* V, const float* log_g,
                               void* O, float* Z,
                               void* workspace, size_t workspace_bytes, void* hip_stream);

pa_status power_attn_bwd_gated(const pa_problem* prob,
                               const void* Q, const void* K, const void* V, const float* log_g,
                               const void* O, const float* Z, const void* dO,
                               void* dQ, void* dK, void* dV, float* dlog_g,
                               void* workspace, size_t workspace_bytes, void* hip_stream);

/* ---- single-token decode step ----------------------------------------------------------------
 * The recurrent form (Sec. 2 Eq. (6)), one iteration per call, with the state kept in device
 * memory between calls (the fixed-cost inference of App. D):
 *     S <- g S + phi(k) [v, 1]^T,    y = S^T phi(scale q),    o = y[:v] / y[v]  (normalize)  or  y[:v]
 * i.e. after n steps on k_1..k_n, v_1..v_n the output equals row n of power_attn_fwd on the same
 * sequence (with the same gates).  Of `prob` the fields B, H, d, v, p, normalize, scale, dtype and
 * gated are used (1 <= p <= 4, d, v <= 128); chunk, impl and keep_state are ignored, and T only by
 * power_attn_decode_absorb.
 *
 * state: DEVICE, caller-owned, power_attn_decode_state_bytes(prob) bytes, float32 inside; it
 * belongs to one (prob, sequence batch) and must be initialised by power_attn_decode_init before
 * the first step (which also builds the index table the steps read).  q, k: DEVICE [B, H, d];
 * v, o: DEVICE [B, H, v], in prob->dtype; z (may be NULL): DEVICE float32 [B, H], the
 * denominator; log_g: DEVICE float32 [B, H], log of this step's gate (<= 0), required when
 * prob->gated, else must be NULL.  Calls are queued on hip_stream and return at once; steps on one
 * state must be ordered by the caller (same stream).  Errors as for the other calls; nothing is
 * launched when validation fails. */
size_t power_attn_decode_state_bytes(const pa_problem* prob);     /* 0 if the problem is invalid or unsupported */
pa_status power_attn_decode_init(const pa_problem* prob, void* state, size_t state_bytes, void* hip_stream);
/* The hand-over from a prompt: updates `state` as prob->T decode steps on K [B, H, T, d], V [B, H, T, v]
 * (log_g [B, H, T] when prob->gated, else NULL) would, without producing their outputs - those are
 * what power_attn_fwd returns for the prompt.  May be called on a state that already holds tokens.
 * workspace (DEVICE, 256-byte aligned, may be NULL): with power_attn_decode_absorb_workspace_bytes(prob)
 * bytes of it (0 = no such path for this problem: bf16, p = 2, d = v = 64, T a multiple of 128 have one)
 * the prompt goes through the matrix-core state scan, some 20x faster, its sums rounded to bf16 once
 * as the chunk states of power_attn_fwd are; without, through a float32 kernel on the vector ALUs. */
size_t power_attn_decode_absorb_workspace_bytes(const pa_problem* prob);
pa_status power_attn_decode_absorb(const pa_problem* prob, const void* K, const void* V, const float* log_g,
                                   void* state, size_t state_bytes, void* workspace, size_t workspace_bytes,
                                   void* hip_stream);
pa_status power_attn_decode_step(const pa_problem* prob, const void* q, const void* k, const void* v,
                                 const float* log_g, void* state, size_t state_bytes,
                                 void* o, float* z, void* hip_stream);

/* The chunk size the calls use for `prob` (prob->chunk itself unless it is 0; 0 on an invalid problem). */
int power_attn_resolved_chunk(const pa_problem* prob);

/* Expanded state rows the chosen kernel family keeps per head for `prob`: C(d+p-1, p) for
 * the generic family (Lemma 4.2), C(d/d_tile+p-1, p) * d_tile^p for the tiled one
 * (Sec. 4.1.1).  0 when no state is built (the attention-form kernels) and on an invalid problem. */
long long power_attn_state_rows(const pa_problem* prob);

const char* power_attn_status_string(pa_status s);

/* Text of the last HIP error that made a call return PA_ERR_HIP ("" if none); HOST string
 * owned by the library, valid until the next failing call. */
const char* power_attn_last_hip_error(void);

/* Destroys the calling host thread's side stream and events (see the top of this file), if it has
 * created any; the next backward call of the thread creates them again.  Call it before a thread that
 * has run power_attn_bwd ends, or not at all (the process's exit releases them). */
void power_attn_release_thread(void);

/* Optional per-kernel timing for benchmarks (a switch per host thread: it records the calls of the
 * thread that turned it on).
 * Between _begin and _end every kernel the library launches is bracketed by a pair of HIP
 * events on the launch stream; _end waits for them and returns, per kernel name, the number
 * of launches and the summed elapsed milliseconds.  `out` is a HOST array of `max_entries`
 * records; the number filled is returned through *n (HOST int).  While the switch is on, the
 * kernels of a call run back to back on the caller's stream (outside it, power_attn_bwd may run
 * independent kernels side by side on a second stream of its own), so that every duration is
 * the kernel's own. */
typedef struct {
    char   name[48];
    int    launches;
    float  ms_total;
} pa_kernel_time;

pa_status power_attn_profile_begin(void);
pa_status power_attn_profile_end(pa_kernel_time* out, int max_entries, int* n);

#ifdef __cplusplus
}
#endif
#endif /* POWER_ATTN_H */
