/*
 * race_attn.h - C ABI of the MI355X (gfx950) RACE Attention library.
 *
 * RACE Attention (arXiv 2510.04008) replaces softmax attention by a linear-time estimator
 * of sharpened angular-kernel attention.  For every head, L independent tables each draw
 * P Gaussian hyperplanes; a query or key x is softly assigned to the R = 2^P corners of
 * the hypercube, phi_r(x) = softmax_r(beta * tanh(W x) . v_r)  (Algorithm 1, steps 2-4);
 * keys and values are accumulated into per-table bucket statistics A = Phi_K^T 1 and
 * B = Phi_K^T V (step 5); every query reads them back, Num = (1/L) sum_l Phi_Q B,
 * Den = (1/L) sum_l Phi_Q A, O = Num / Den (steps 7-8).  The causal variant
 * (Algorithm 2, appendix "Causal RACE Attention") lets query t read the statistics of
 * keys 1..t only (inclusive: token t is added before it reads).
 *
 * Conventions common to all entry points
 *   - Tensors Q, K, V, O, dO, dQ, dK, dV are DEVICE pointers to (B, H, N, d) arrays,
 *     row-major with d contiguous, of the element type named by desc->dtype.
 *     den is a DEVICE pointer to (B, H, N) float.  Buffers must not overlap.
 *   - proj_seeds is a HOST pointer to H 64-bit seeds, one per head, read during the call.
 *     W is shared by the batch.  Head h uses the (L*P, d) matrix whose row l*P+t is
 *     hyperplane t of table l, drawn i.i.d. N(0,1) (Algorithm 1, step 2) by the generator
 *     documented at race_attn_expand_projection().
 *   - Corner r of the hypercube has v_{r,t} = +1 iff bit t of r is set (t = 0 is the least
 *     significant bit and belongs to row l*P+0 of W).
 *   - sharpening is the temperature beta of Algorithms 1/2.  Q and K are used as given:
 *     no 1/sqrt(d) scaling happens inside the layer, and no normalisation unless desc->unit_qk
 *     asks for it.  With unit_qk = 1 every entry point that hashes rows of Q or K (passes, taps,
 *     state_init, step) uses x / max(|x|, 1e-12) in place of the row x, in fp32 from the stored
 *     elements; the backward passes carry the chain rule through that map, (I - xhat xhat^T) / |x|.
 *     beta = +infinity selects the hard hash h(x) = sign(W x) that Section 3.3 starts from
 *     (bit t of the bucket is [<w_t, x> >= 0]; counters instead of soft masses), for inference:
 *     the forward pass, the taps and incremental decoding accept it, the backward passes return
 *     RACE_ERR_UNSUPPORTED (the hard hash is piecewise constant).  A query all of whose buckets
 *     are empty has den = 0 and gets O = 0 (non-causal only; the soft layer never has den = 0).
 *   - The caller owns every buffer, including the workspace (device memory, 256-byte
 *     aligned, at least race_attn_workspace_bytes() bytes; contents are scratch).  The
 *     library allocates no device memory, never synchronises the stream and launches all
 *     work on the given stream.  Calls that share a workspace must be stream-ordered.
 *   - The host keeps one pinned image of the packed W per distinct (proj_seeds, H, d, L, P, dtype) for the life of
 *     the process (asynchronous copies and captured graphs may read it at any time; a few KB to ~100 KB each).
 *     The 4097th distinct combination in one process is refused with RACE_ERR_HIP.
 *   - Every argument is checked before anything is launched; on any error status other
 *     than RACE_ERR_HIP the outputs are untouched.  N == 0 is a valid no-op.
 *   - Arithmetic: products of bf16 operands are accumulated in fp32; the fp32 element
 *     type computes in fp32 throughout.
 */
#ifndef RACE_ATTN_H
#define RACE_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    RACE_OK = 0,
    RACE_ERR_INVALID_ARG = 1, /* null pointer, non-positive size, non-finite beta, bad enum   */
    RACE_ERR_UNSUPPORTED = 2, /* a valid shape outside what the kernels were built for         */
    RACE_ERR_WORKSPACE = 3,   /* workspace null, misaligned or smaller than required           */
    RACE_ERR_HIP = 4,         /* a HIP call failed; text from race_attn_last_error()           */
    RACE_ERR_NOT_READY = 5    /* a call that prepares this one has not been made (see the entry
                                 point); text from race_attn_last_error()                       */
} race_status_t;

typedef enum { RACE_F32 = 0, RACE_BF16 = 1 } race_dtype_t;

/* ABI-identical to hipStream_t (a pointer to HIP's opaque stream object); 0 = default stream. */
typedef struct ihipStream_t *race_stream_t;

/* Problem statement of Algorithms 1/2: inputs Q, K, V in R^{N x d}, L tables, P hyperplanes,
 * temperature beta; batched over (B, H). */
typedef struct {
    int32_t B, H;     /* batch, heads (>= 1)                                                   */
    int64_t N;        /* tokens per sequence (>= 0)                                            */
    int32_t d;        /* head dimension: multiple of 8, 8 <= d <= 256                          */
    int32_t L, P;     /* tables (>= 1), hyperplanes per table (1..8); R = 1 << P               */
    float sharpening; /* beta > 0; +infinity = hard hash (forward only)                        */
    int32_t causal;   /* 0: Algorithm 1 (all keys); 1: Algorithm 2 (keys j <= i)               */
    int32_t dtype;    /* race_dtype_t of Q, K, V, O, dO, dQ, dK, dV                            */
    int64_t chunk;    /* tokens per scan segment: the sequence is cut into segments whose
                         bucket statistics are combined by a prefix scan; 0 = choose           */
    int32_t unit_qk;  /* 0: Q and K enter the projection as given (Algorithm 1, step 4);
                         1: every row of Q and K is first divided by its Euclidean norm, the
                         setting |Q_i| = |K_j| = 1 of Theorem 1's proof (Appendix, "Setup and
                         assumptions"); dQ and dK are then the cotangents of the rows as given  */
} race_attn_desc_t;

/* Bytes of device workspace that race_attn_fwd / race_attn_bwd / race_attn_debug_buckets need
 * for this descriptor (one figure covers all three).  Returns 0 for an invalid or unsupported
 * descriptor (and for N == 0). */
size_t race_attn_workspace_bytes(const race_attn_desc_t *desc);

/* Forward pass, Algorithm 1 (causal == 0) or Algorithm 2 (causal == 1).
 * in : Q, K, V (device), proj_seeds (host, H entries)
 * out: O (device, same type as V), den (device, float (B,H,N)): Den_i including the 1/L of
 *      Algorithm 1 step 7; the backward pass needs O and den. */
race_status_t race_attn_fwd(const race_attn_desc_t *desc, const void *Q, const void *K, const void *V,
                            const uint64_t *proj_seeds, void *O, float *den,
                            void *workspace, size_t workspace_bytes, race_stream_t stream);

/* For callers that cannot allocate (code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): race_attn_fwd without a workspace argument.  The kernels are race_attn_fwd's; their scratch (the
 * packed W and the per-segment bucket statistics) lives in an array of 32 MiB that is part of the library's code
 * object, one copy per GPU, held until the process ends.  The call allocates nothing, on the host or on the device.
 *   - Size limit: if the workspace race_attn_fwd would use exceeds the array, the sequence is cut into fewer, longer
 *     scan segments (desc->chunk doubled as often as needed; O and den then differ from race_attn_fwd's by the
 *     rounding of a different summation order only); a problem that does not fit even as one segment per
 *     (batch, head) returns RACE_ERR_WORKSPACE.  At d = 128, L = 8, P = 6 (bf16) a segment's statistics take 258 KiB
 *     and the hashed rows of Q and K 384 bytes per token and head: B*H*(segments * 258 KiB + N * 384 B) < 32 MiB.
 *   - The pinned host image of W for (proj_seeds, shape) must exist already, because making it allocates: any
 *     earlier call of another entry point with the same H, d, L, P, dtype and proj_seeds (race_attn_fwd,
 *     race_attn_debug_hash, ...) leaves it in the library's host cache for the life of the process.  Otherwise
 *     RACE_ERR_NOT_READY, and nothing is launched.
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different streams or
 *     threads) race; stream-ordered calls are fine.  Nothing in the array needs clearing between calls (every
 *     element read by a kernel has been written earlier in the same call).
 * Everything else (arguments, outputs, errors) is as for race_attn_fwd.  There is no race_attn_bwd_saved on this
 * scratch: the next call overwrites it. */
race_status_t race_attn_fwd_static(const race_attn_desc_t *desc, const void *Q, const void *K, const void *V,
                                   const uint64_t *proj_seeds, void *O, float *den, race_stream_t stream);

/* Backward pass of the same operator: given dO = d(loss)/dO, O and den from race_attn_fwd on the
 * same inputs, writes dQ, dK, dV.  The paper trains through the differentiable soft assignment
 * (Section 3.3) and prints no gradient; the formulas are the chain rule through Algorithms 1/2:
 * read-out, bucket accumulation (a suffix scan in the causal case), corner softmax, tanh and W.
 * W is a fixed random matrix and gets no gradient. */
race_status_t race_attn_bwd(const race_attn_desc_t *desc, const void *Q, const void *K, const void *V,
                            const void *O, const float *den, const void *dO,
                            const uint64_t *proj_seeds, void *dQ, void *dK, void *dV,
                            void *workspace, size_t workspace_bytes, race_stream_t stream);

/* The same backward pass, which also returns the cotangent of the temperature: the paper's experiments train
 * beta (Section 4), and with W fixed and random it is the layer's only parameter.  The corner logits of Algorithm 1, step 4 are beta * (tanh(W x) . v_r), so
 * d(loss)/d(beta) = sum over Q and K tokens, tables and corners of dlogit_r * (tanh(W x) . v_r).
 * dbeta: DEVICE float (B, H), one partial derivative per (batch, head), written (not accumulated); the
 * derivative with respect to a beta shared by all of them is the sum of the entries.  NULL = not wanted, which
 * makes this call identical to race_attn_bwd.  Sums are formed in a fixed order (bit-reproducible).  Needs no
 * more workspace than race_attn_bwd.  N == 0 writes nothing. */
race_status_t race_attn_bwd_beta(const race_attn_desc_t *desc, const void *Q, const void *K, const void *V,
                                 const void *O, const float *den, const void *dO,
                                 const uint64_t *proj_seeds, void *dQ, void *dK, void *dV, float *dbeta,
                                 void *workspace, size_t workspace_bytes, race_stream_t stream);

/* The backward pass for a caller that kept the forward's workspace.  race_attn_fwd leaves in the workspace what
 * the backward pass would otherwise derive again from Q, K and V: the packed W, the hashed rows of Q and K (one
 * float per token, table and hyperplane: all that the soft assignment of Algorithm 1, step 4 depends on) and the
 * key/value bucket statistics (A, B of Algorithm 1, step 5; in the causal case Algorithm 2's running statistics at
 * the start of every scan segment).  This entry point reads them instead of recomputing them: one projection pass
 * over Q and K and one accumulation pass over K and V fewer.
 * Contract: `workspace` is the buffer that the last race_attn_fwd with the same desc, Q, K, V and proj_seeds wrote,
 * nothing has written to it since, and this call is stream-ordered after that forward.  A workspace that does not
 * hold that forward's data gives wrong gradients, never an out-of-bounds access.  Arguments, outputs, dbeta
 * (may be NULL) and error behaviour are those of race_attn_bwd_beta, whose results it reproduces bit for bit.
 * Kernel families that keep no such statistics recompute them (the call is then race_attn_bwd_beta). */
race_status_t race_attn_bwd_saved(const race_attn_desc_t *desc, const void *Q, const void *K, const void *V,
                                  const void *O, const float *den, const void *dO,
                                  const uint64_t *proj_seeds, void *dQ, void *dK, void *dV, float *dbeta,
                                  void *workspace, size_t workspace_bytes, race_stream_t stream);

/* Host-only: expands the seeds into W_host (HOST, float, (H, L*P, d)), the values the kernels
 * multiply with (Algorithm 1, step 2).  Generator: element e = row*d + col of head h is Gaussian
 * number (e mod 4) of block e/4 of Philox-4x32-10 with key = (low, high) 32 bits of the head's
 * seed and counter = (block low, block high, 0, 0); the block's words (x0,x1,x2,x3) give
 * Box-Muller pairs from (x0,x1) and (x2,x3) with u = (x + 0.5) / 2^32, evaluated in fp64:
 * sqrt(-2 ln u1) * (cos, sin)(2 pi u2); rounded to fp32 (nearest even), and for RACE_BF16 once
 * more to bf16 (nearest even, returned widened to float).  Only H, L, P, d, dtype of desc are used. */
race_status_t race_attn_expand_projection(const race_attn_desc_t *desc, const uint64_t *proj_seeds,
                                          float *W_host);

/* Debug tap of the projection and soft assignment (Algorithm 1, steps 2-4) of one tensor X (Q or K):
 * codes (device, uint8 (B,H,N,L)): bit t = [<w_t, x> >= 0], i.e. the hard hash sign(W x) of
 * Section 3.3, which is also the arg-max corner of phi;  phi (device, float (B,H,N,L,R)) or NULL.
 * Runs the projection arithmetic of the production kernels.  Needs no workspace beyond
 * H*L*P*d floats + 256 bytes. */
race_status_t race_attn_debug_hash(const race_attn_desc_t *desc, const void *X, const uint64_t *proj_seeds,
                                   uint8_t *codes, float *phi,
                                   void *workspace, size_t workspace_bytes, race_stream_t stream);

/* Debug tap of the bucket statistics of Algorithm 1, step 5, over all N keys (whatever causal
 * says): A (device, float (B,H,L,R)) and Bsum (device, float (B,H,L,R,d)). */
race_status_t race_attn_debug_buckets(const race_attn_desc_t *desc, const void *K, const void *V,
                                      const uint64_t *proj_seeds, float *A, float *Bsum,
                                      void *workspace, size_t workspace_bytes, race_stream_t stream);

/* ---- Incremental decoding: the bucket statistics as the carried state (Algorithm 2, one loop iteration per
 * call).  The state plays the part of a key/value cache whose size does not grow with the context:
 * state = DEVICE float (B, H, L, R, d+1), row-major; per bucket row the d sums of phi_K * V (B of Algorithm 1,
 * step 5) followed by the mass (A).  The caller owns it; a zero-filled state is the empty context. */

/* Bytes of one state for this descriptor (B, H, d, L, P are used); 0 for an invalid descriptor. */
size_t race_attn_state_bytes(const race_attn_desc_t *desc);

/* Prefill: state <- statistics of the desc->N keys and values in K, V (DEVICE (B, H, N, d) of desc->dtype);
 * N == 0 zero-fills it.  Workspace as for race_attn_fwd (race_attn_workspace_bytes; none needed for N == 0). */
race_status_t race_attn_state_init(const race_attn_desc_t *desc, const void *K, const void *V,
                                   const uint64_t *proj_seeds, float *state,
                                   void *workspace, size_t workspace_bytes, race_stream_t stream);

/* Bytes of device workspace race_attn_step needs (independent of desc->N). */
size_t race_attn_step_workspace_bytes(const race_attn_desc_t *desc);

/* One new token per (batch, head): q, k, v are DEVICE (B, H, d) rows of desc->dtype.  The state is updated in
 * place with (k, v) first, then q reads it (the loop body of Algorithm 2): o (DEVICE (B, H, d), desc->dtype) and
 * den (DEVICE float (B, H), with the 1/L of Algorithm 1 step 7).  desc->N, desc->causal and desc->chunk are
 * ignored.  Arithmetic is fp32 on the values as given.  Cost O(L R d) per token and head; one kernel launch.
 * The call expands proj_seeds into the workspace (a copy from pinned host memory) and leaves W there: a later step
 * with the same desc on a workspace nobody has written to since may pass proj_seeds = NULL and skips the copy. */
race_status_t race_attn_step(const race_attn_desc_t *desc, const void *q, const void *k, const void *v,
                             const uint64_t *proj_seeds, float *state, void *o, float *den,
                             void *workspace, size_t workspace_bytes, race_stream_t stream);

/* Static, never-null description of a status code. */
const char *race_status_string(race_status_t status);

/* Text of the most recent failure that has one, as seen by the calling thread ("" if none): the HIP error behind
 * RACE_ERR_HIP, the reason for RACE_ERR_NOT_READY, the limit behind race_attn_fwd_static's RACE_ERR_WORKSPACE. */
const char *race_attn_last_error(void);

/* Which kernel family a descriptor is served by: 0 = invalid/unsupported, 1 = generic fp32-math
 * kernels, 2 = bf16 MFMA kernels.  Informational (benchmarks and tests report it).
 * The generic kernels serve fp32 tensors and every bf16 shape without an MFMA instantiation; they keep per-table
 * partial results of every token in the workspace (3 * B*H*L*N*d floats for the backward pass), and a descriptor whose
 * partial results would exceed 16 GiB is RACE_ERR_UNSUPPORTED (e.g. fp32, d = 64, L = 4: B*H*N beyond 5.6 million).
 * Test switch: with RACE_ATTN_FORCE_GENERIC=1 in the environment every descriptor is planned on the generic kernels
 * (the tests use it to run one problem on both families; it is read at every call). */
int race_attn_kernel_family(const race_attn_desc_t *desc);

/* Tokens per scan segment the library uses for this descriptor (desc->chunk rounded to what the kernels take, or
 * the library's own choice for chunk = 0): segment s covers tokens [s * len, min(N, (s + 1) * len)), and the
 * statistics at segment boundaries are what the prefix scan of Algorithm 2's cumulative arrays hands from one
 * workgroup to the next.  Informational (tests place their windows across these boundaries).  0 = invalid. */
int64_t race_attn_segment_tokens(const race_attn_desc_t *desc);

/* Benchmark aid (no passage of the paper; callers: benchmarks and profilers).  While enabled for the
 * calling thread, every kernel the library launches is bracketed by a pair of HIP events recorded on the
 * call's own stream.  race_attn_profile_read() waits for the recorded events, adds up the elapsed time per
 * kernel name since the previous read, writes up to max_entries results (names are static strings, total_ms
 * in milliseconds, launches = number of launches) and returns how many distinct kernels ran.  Enabling
 * creates HIP events (host allocations); results are discarded by disabling. */
void race_attn_profile_enable(int on);
int race_attn_profile_read(int max_entries, const char **names, float *total_ms, int *launches);

/* Benchmark aid (no passage of the paper; callers: counter calibration).  Copies `bytes` bytes (a multiple
 * of 16) from src to dst (DEVICE pointers, 16-byte aligned, not overlapping) with one plain grid-stride kernel
 * named calibration_copy_kernel that reads every byte once and writes every byte once: a dispatch of known HBM
 * traffic against which hardware byte counters of the other kernels are scaled.  bytes == 0 is a no-op. */
race_status_t race_attn_calibration_copy(void *dst, const void *src, size_t bytes, race_stream_t stream);

/* Benchmark aid (no passage of the paper; callers: benchmarks that report the attainable matrix rate next to the
 * published peak).  Launches calibration_mfma_kernel: `workgroups` workgroups of 256 threads, each wavefront
 * issuing `iters` rounds of four independent v_mfma_f32_32x32x16_bf16 on register operands, i.e.
 * workgroups * 4 * iters * 4 * 32768 floating-point operations in all; every lane then stores one float to
 * sink (DEVICE, workgroups * 256 floats) so that the work cannot be optimised away.  vector_ops (0, 4, 8 or 16):
 * that many independent v_mul_f32 on registers of the same wavefront follow every matrix instruction, which
 * measures how much vector work the matrix pipeline hides (the flop count returned by the binding counts the
 * matrix instructions only).  workgroups and iters must be in 1 .. 2^20. */
race_status_t race_attn_calibration_mfma(int workgroups, int iters, int vector_ops, float *sink, race_stream_t stream);

#ifdef __cplusplus
}
#endif
#endif /* RACE_ATTN_H */
