/*
 * la.h: C ABI of the MI355X (gfx950) linear-attention library.
 *
 * Kernelised attention with the feature map phi(x) = elu(x) + 1 (paper eq. 7):
 * causal forward (eq. 9-12), its constant-memory backward (eq. 13-15,
 * Algorithm 1), the non-causal forward (eq. 4-6) and the recurrent decode step
 * (eq. 16-20).
 *
 * Conventions shared by every entry point
 *   Pointers   All tensor pointers are DEVICE pointers (HBM) valid on the
 *              current HIP device.  The library never allocates, frees or keeps
 *              them; the caller owns every buffer including the workspace.
 *   Layout     Dense row-major [B, H, N, D] (Q, K and their gradients) and
 *              [B, H, N, M] (V, O and their gradients): each (batch, head) pair
 *              is one contiguous N x D slab and an independent problem.
 *   dtype      `t` is the element type of the N-sized tensors only (Q, K, V, O,
 *              dO, dQ, dK, dV; q, k, v, out in the step).  den, the workspace,
 *              the decode state S, z and all accumulation are always fp32.
 *              LA_BF16 tensors hold raw bfloat16 bit patterns (uint16).
 *   Feature map phi(x) = elu(x) + 1 (eq. 7) is applied to Q and K inside every
 *              call, and dQ, dK are gradients with respect to the raw Q, K.
 *              With t = LA_F32_FEATURES / LA_BF16_FEATURES the caller has
 *              applied a feature map of its own (section 3.2 allows any map
 *              with non-negative values; Algorithm 1 is stated on mapped
 *              inputs): Q and K (q and k of the decode calls) then hold the
 *              feature values, no map is applied, and dQ, dK are gradients
 *              with respect to those features.  The feature width is D.
 *              With t = LA_F32_POLY2 the feature map is that of the polynomial
 *              kernel of degree 2 (section 3.2), sim(q, k) = (q . k)^2:
 *              phi(x) = vec(x x^T), feature D*i + j = x_i x_j.  Q and K (q, k of the
 *              decode calls) hold the RAW vectors, D = 8 values per token (fp32),
 *              the kernels build the C = D^2 = 64 features as they load a tile
 *              (a call reads 32 bytes of Q per token and head, not 256), and dQ, dK
 *              are gradients with respect to the raw vectors, [.., 8] like Q and K.
 *              Everything sized by the feature width is sized by C: the decode
 *              state S [B,H,C,M], z [B,H,C] and the states of the _state entry
 *              points.  The features are signed, so den is not bounded away from
 *              zero by construction: pass an eps that suits the data.  All entry
 *              points take this code.
 *   Sizes      B, H, N >= 1.  N needs no alignment.  D and M must each be 32 or
 *              64 (LA_ERR_UNSUPPORTED otherwise; LA_F32_POLY2: D = 8, M 32 or 64).
 *              B*H*N*max(D,M) < 2^40.
 *   eps        den_i = phi(Q_i) . Z_i + eps, added once to the finished dot
 *              product; eps >= 0.  With eps = 0 a denominator can still be exactly
 *              0 in fp32: phi(x) = exp(x) underflows to 0 for x below about -87, and
 *              if that holds for every key up to a token (or for all of its
 *              queries), its output and the gradients that pass through it are
 *              not finite.  Pass eps > 0 where inputs that negative can occur.
 *   Stream     `stream` is a hipStream_t passed as void*; NULL is the default
 *              stream.  Every call only enqueues work and returns without
 *              synchronising.
 *   Alignment  Tensor pointers must be 16-byte aligned (LA_ERR_ALIGN).
 *   Errors     Return value: LA_OK (0) or a negative la_status.  Argument
 *              errors are detected on the host before anything is launched;
 *              a failed launch returns LA_ERR_HIP.  No exceptions, no abort.
 *   Aliasing   A buffer that a call writes (outputs, workspace, the decode state)
 *              must not overlap any other buffer of the call: LA_ERR_ALIAS,
 *              checked on the host from the pointers and the sizes, last of
 *              the argument checks.
 *   Determinism No floating-point atomics: the same call on the same inputs
 *              gives bit-identical results.
 *   Non-finite Inf or NaN in the inputs gives unspecified results, with one
 *              guarantee: the causal forward's outputs and denominators before
 *              token t do not depend on what Q, K, V hold from token t on,
 *              finite or not (the causal mask of eq. 8).
 *   Threads    No global mutable state apart from the tuning values below and
 *              la_causal_fwd_noalloc's built-in scratch array; calls from
 *              several host threads are safe as long as they do not share
 *              output or workspace buffers.
 *   Tuning     Five environment variables override the schedule (for tests and
 *              experiments): LA_TARGET_WAVES (default 2048: wavefronts wanted
 *              in flight), LA_MIN_SEG_CHUNKS (default 2: shortest segment, in
 *              16-token chunks), LA_FOLD_MAX_SEGS (default 8: up to this many
 *              segments per sequence the passes add up the segment totals
 *              themselves and no scan kernel runs), LA_BWD_SEG_GROUP (1 or 2:
 *              how many of the forward's segments a workgroup of the backward
 *              takes; default 1 for 32 x 32 heads, else 2) and LA_STREAM_LOADS
 *              (1: non-temporal instead of plain loads of the tensors).
 *              Sequences are not cut at all once B*H reaches half of
 *              LA_TARGET_WAVES.  The environment is read once per process, by
 *              the first workspace query or entry point, so a query and the
 *              calls that use its workspace see the same values;
 *              la_tuning_reload() reads it again.
 */
#ifndef LA_H_
#define LA_H_

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LA_F32 = 0,
    LA_BF16 = 1,
    LA_F32_FEATURES = 2,      /* fp32, Q and K hold feature values already  */
    LA_BF16_FEATURES = 3,     /* bf16, Q and K hold feature values already  */
    LA_F32_POLY2 = 4          /* fp32, degree-2 polynomial kernel: phi(x) = vec(x x^T)  */
} la_dtype;

typedef enum {
    LA_OK = 0,
    LA_ERR_NULL = -1,         /* a required pointer is NULL                         */
    LA_ERR_SHAPE = -2,        /* B, H or N < 1, eps < 0 or not finite, size overflow */
    LA_ERR_UNSUPPORTED = -3,  /* D or M not in {32, 64} (LA_F32_POLY2: D != 8), unknown dtype */
    LA_ERR_WORKSPACE = -4,    /* ws is NULL or ws_bytes is smaller than the query   */
    LA_ERR_HIP = -5,          /* a HIP call or kernel launch failed                 */
    LA_ERR_ALIGN = -6,        /* a tensor pointer is not 16-byte aligned            */
    LA_ERR_ALIAS = -7,        /* a written buffer overlaps another buffer of the call */
    LA_ERR_SCRATCH = -8       /* la_causal_fwd_noalloc: the sizes need more than the built-in scratch */
} la_status;

/* Static, NUL-terminated description of a status code. */
const char *la_status_string(int status);

/* Library version, major * 10000 + minor * 100 + patch. */
int la_version(void);

/*
 * Reads the tuning variables of the environment again (see "Tuning" above).
 * For tests and experiments that change them inside a process.  Not to be
 * called while another thread is inside an entry point or between a workspace
 * query and the calls that rely on it.
 */
void la_tuning_reload(void);

/*
 * Workspace queries.  Host-only, no GPU call.  Return the number of bytes the
 * matching entry point needs for these sizes on the current device (0 is
 * possible: then ws may be NULL), or 0 for invalid sizes (the entry point
 * itself reports the error).  The workspace holds per-segment partial states
 * (the running sums of eq. 10-11 cut at segment borders, so that one long
 * sequence can occupy many compute units) and, for the backward, three fp32
 * scalars per token (1/den, the gradient that reaches den, and room for den
 * itself when the caller does not pass it): no N x M buffer.
 */
size_t la_causal_fwd_workspace(int B, int H, int N, int D, int M, la_dtype t);
size_t la_causal_bwd_workspace(int B, int H, int N, int D, int M, la_dtype t);
size_t la_global_fwd_workspace(int B, int H, int N, int D, int M, la_dtype t);
size_t la_global_bwd_workspace(int B, int H, int N, int D, int M, la_dtype t);

/*
 * Causal linear attention, forward (eq. 9 in its prefix-sum form eq. 10-12):
 *   S_i = sum_{j<=i} phi(K_j) V_j^T,  Z_i = sum_{j<=i} phi(K_j),
 *   den_i = phi(Q_i) . Z_i + eps,     O_i = phi(Q_i)^T S_i / den_i.
 * Q, K [B,H,N,D] in; V [B,H,N,M] in; O [B,H,N,M] out; den [B,H,N] fp32 out or
 * NULL (pass it if la_causal_bwd will follow).  ws: la_causal_fwd_workspace()
 * bytes of scratch, contents undefined before and after.
 */
int la_causal_fwd(const void *Q, const void *K, const void *V, void *O, float *den,
                  int B, int H, int N, int D, int M, float eps, la_dtype t,
                  void *ws, size_t ws_bytes, void *stream);

/*
 * la_causal_fwd for callers that cannot allocate device memory or must not call anything that
 * does: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, results (bit for bit) and schedule as la_causal_fwd, minus the workspace:
 * the per-segment running sums live in an array of LA_NOALLOC_SCRATCH_BYTES that is part of
 * the library's own device code (every GPU the library runs on holds one copy until the
 * process ends).  The call itself allocates and frees nothing and calls no allocating routine;
 * the first call on a device looks the array's address up (make that call outside a graph
 * capture).  Sizes whose la_causal_fwd_workspace() exceeds LA_NOALLOC_SCRATCH_BYTES are refused
 * with LA_ERR_SCRATCH before anything is launched (the metric's shape, B=2, H=8, N=65536,
 * D=M=64, needs 32.5 MiB and fits).  All calls on one GPU share that GPU's array, which keeps
 * whatever the last call left in it (nothing in it needs clearing: a call writes every slot
 * before reading it): calls that overlap in time on one GPU, from any thread or stream, race;
 * serialise them on one stream or with events.  The caller still owns Q, K, V, O, den.
 */
#define LA_NOALLOC_SCRATCH_BYTES ((size_t)40 << 20)
int la_causal_fwd_noalloc(const void *Q, const void *K, const void *V, void *O, float *den,
                          int B, int H, int N, int D, int M, float eps, la_dtype t, void *stream);

/*
 * The same forward with the recurrent state handed in and out (eq. 16-19 seen from the
 * parallel side): S0 [B,H,D,M], z0 [B,H,D] fp32 are the state before token 0 (both NULL: zero,
 * eq. 16-17), S1, z1 receive the state after token N-1 (both NULL: not wanted).  A prompt can
 * be processed in parallel and continued token by token with la_recurrent_step, or a long
 * sequence processed in pieces.  S0/z0 must not alias S1/z1.  Workspace as la_causal_fwd.
 */
int la_causal_fwd_state(const void *Q, const void *K, const void *V, const float *S0,
                        const float *z0, void *O, float *den, float *S1, float *z1,
                        int B, int H, int N, int D, int M, float eps, la_dtype t,
                        void *ws, size_t ws_bytes, void *stream);
/* The same on token-major tensors (see la_causal_fwd_bnhd): Q, K [B,N,H,D], V, O [B,N,H,M];
 * den [B,H,N] and the states [B,H,D,M], [B,H,D] keep their layouts. */
int la_causal_fwd_state_bnhd(const void *Q, const void *K, const void *V, const float *S0,
                             const float *z0, void *O, float *den, float *S1, float *z1,
                             int B, int H, int N, int D, int M, float eps, la_dtype t,
                             void *ws, size_t ws_bytes, void *stream);

/*
 * Causal linear attention, backward (eq. 13-15 / Algorithm 1 applied to the
 * numerator and to the denominator together, then the chain rule through phi):
 * given dO = dL/dO it writes dQ, dK (with respect to the RAW Q, K, i.e.
 * through phi) and dV.  One forward and one reverse cumulative sum; memory is
 * O(N max(D,M)), no per-position state is stored.
 * den [B,H,N] is the denominator output of la_causal_fwd on the same Q, K, V,
 * eps; NULL: the forward is recomputed into the workspace.  O is NOT read and
 * may be NULL (a caller need not keep it for the backward): the one place the
 * gradient needs it, dO_i . O_i, equals phi(Q_i) . (S_i dO_i)/den_i, which the
 * dQ pass has at hand.  The argument stays for symmetry with the forward.
 * fwd_ws is optional (NULL allowed): the workspace that la_causal_fwd used for
 * that same call, untouched since.  It then still holds the running sums of
 * eq. 10-11 at the segment borders, and the backward reuses them instead of
 * re-reading K and V to rebuild them (one state per segment of a few hundred
 * tokens, not one per position).  Must come from the same sizes, dtype and
 * schedule; ignored when the sizes need no forward workspace.
 * dQ, dK [B,H,N,D] out; dV [B,H,N,M] out.  ws as above
 * (la_causal_bwd_workspace()).
 */
int la_causal_bwd(const void *Q, const void *K, const void *V, const void *O, const float *den,
                  const void *fwd_ws, const void *dO, void *dQ, void *dK, void *dV,
                  int B, int H, int N, int D, int M, float eps, la_dtype t,
                  void *ws, size_t ws_bytes, void *stream);

/*
 * The same backward for a piece of a sequence whose recurrent state was handed in
 * and out by la_causal_fwd_state (backpropagation through time for the RNN of
 * eq. 16-20, section 3.4).  S0, z0: the state before token 0 that the forward
 * started from (both NULL: zero).  dS1 [B,H,D,M], dz1 [B,H,D] fp32 in: gradient
 * of the loss with respect to the state after token N-1, from whatever consumed
 * that state (both NULL: zero); it is the starting value of the reverse sum of
 * eq. 14-15.  dS0, dz0 fp32 out (both NULL: not wanted): gradient with respect
 * to (S0, z0), i.e. the reverse sum after token 0, to be handed to the piece
 * before as its dS1, dz1.  Pieces chained this way reproduce the gradients of
 * the uncut sequence.  O, den, fwd_ws: results (and workspace) of
 * la_causal_fwd_state with the same S0, z0; den NULL: recomputed; O not read.  The
 * in-buffers must not alias the out-buffers.  Workspace as la_causal_bwd.
 */
int la_causal_bwd_state(const void *Q, const void *K, const void *V, const float *S0,
                        const float *z0, const void *O, const float *den, const void *fwd_ws,
                        const void *dO, const float *dS1, const float *dz1, void *dQ, void *dK,
                        void *dV, float *dS0, float *dz0, int B, int H, int N, int D, int M,
                        float eps, la_dtype t, void *ws, size_t ws_bytes, void *stream);
/* The same on token-major tensors: Q, K, dQ, dK [B,N,H,D]; V, O, dO, dV [B,N,H,M]; den and
 * the state tensors keep their layouts; O, den, fwd_ws from la_causal_fwd_state_bnhd. */
int la_causal_bwd_state_bnhd(const void *Q, const void *K, const void *V, const float *S0,
                             const float *z0, const void *O, const float *den, const void *fwd_ws,
                             const void *dO, const float *dS1, const float *dz1, void *dQ, void *dK,
                             void *dV, float *dS0, float *dz0, int B, int H, int N, int D, int M,
                             float eps, la_dtype t, void *ws, size_t ws_bytes, void *stream);

/*
 * la_causal_fwd and la_causal_bwd on tensors laid out [B,N,H,.] (token-major, the heads of a
 * token side by side: what a fused projection x W_Q of eq. 1 / eq. 20 produces and what the
 * output projection consumes), so that a model need not transpose Q, K, V, O and their
 * gradients into [B,H,N,.] and back.  Q, K, dQ, dK [B,N,H,D]; V, O, dO, dV [B,N,H,M].  The
 * per-token scalars keep their layout: den [B,H,N] fp32.  Everything else (meaning of the
 * arguments, workspace sizes and queries, fwd_ws, O not read, errors) as for la_causal_fwd /
 * la_causal_bwd; a forward and its backward must use the same layout.  A row of one head is
 * D (or M) contiguous elements, rows of a sequence are H * D elements apart: the kernels
 * fetch the same 16-token tiles as 16 such rows.
 */
int la_causal_fwd_bnhd(const void *Q, const void *K, const void *V, void *O, float *den,
                       int B, int H, int N, int D, int M, float eps, la_dtype t,
                       void *ws, size_t ws_bytes, void *stream);
int la_causal_bwd_bnhd(const void *Q, const void *K, const void *V, const void *O, const float *den,
                       const void *fwd_ws, const void *dO, void *dQ, void *dK, void *dV,
                       int B, int H, int N, int D, int M, float eps, la_dtype t,
                       void *ws, size_t ws_bytes, void *stream);

/*
 * Non-causal linear attention, forward (eq. 5-6): the sums over all N keys are
 * formed once and reused for every query,
 *   O_i = phi(Q_i)^T (sum_j phi(K_j) V_j^T) / (phi(Q_i) . sum_j phi(K_j) + eps).
 * Arguments as la_causal_fwd; den [B,H,N] fp32 out (the denominators, eps
 * included) or NULL.  ws: la_global_fwd_workspace() bytes (never 0).
 * Sequences shorter than N in one batch: give the K rows of the padded tokens
 * the value -inf (phi(-inf) = 0 and phi'(-inf) = 0 exactly, so they drop out of
 * both sums) and, in the backward, the dO rows of the padded queries zeros.
 */
int la_global_fwd(const void *Q, const void *K, const void *V, void *O, float *den,
                  int B, int H, int N, int D, int M, float eps, la_dtype t,
                  void *ws, size_t ws_bytes, void *stream);

/*
 * Non-causal linear attention, backward: the gradient of eq. 4-6 for Q, K, V
 * given dO.  With no mask both sums of the causal gradients (eq. 13-15) run
 * over the whole sequence, so with the ones-augmented values of the causal
 * backward (V~ = [V, 1], G~_i = [dO_i/den_i, -(dO_i.O_i)/den_i]) and the two
 * totals S~ = sum_j phi(K_j) V~_j^T and R~ = sum_i phi(Q_i) G~_i^T,
 *   dphi(Q)_i = S~ G~_i,   dphi(K)_j = R~ V~_j,   dV_j = (R~^T phi(K_j))[0:M],
 * followed by the chain rule through phi (elementwise times phi'(Q), phi'(K)).
 * den is the denominator output of la_global_fwd on the same Q, K, V, eps
 * (NULL: recomputed into the workspace); O is not read and may be NULL, as in
 * la_causal_bwd.  fwd_ws is optional
 * (NULL allowed): the workspace la_global_fwd used for that call, untouched
 * since; it still holds S~ and the backward then does not re-read K and V to
 * rebuild it.  dQ, dK [B,H,N,D] out; dV [B,H,N,M] out.  ws:
 * la_global_bwd_workspace() bytes.  Errors as the other entry points.
 */
int la_global_bwd(const void *Q, const void *K, const void *V, const void *O, const float *den,
                  const void *fwd_ws, const void *dO, void *dQ, void *dK, void *dV,
                  int B, int H, int N, int D, int M, float eps, la_dtype t,
                  void *ws, size_t ws_bytes, void *stream);

/*
 * la_global_fwd and la_global_bwd on token-major tensors [B,N,H,.] (see la_causal_fwd_bnhd):
 * Q, K, dQ, dK [B,N,H,D]; V, O, dO, dV [B,N,H,M]; den [B,H,N] fp32.  Everything else as for
 * la_global_fwd / la_global_bwd.
 */
int la_global_fwd_bnhd(const void *Q, const void *K, const void *V, void *O, float *den,
                       int B, int H, int N, int D, int M, float eps, la_dtype t,
                       void *ws, size_t ws_bytes, void *stream);
int la_global_bwd_bnhd(const void *Q, const void *K, const void *V, const void *O, const float *den,
                       const void *fwd_ws, const void *dO, void *dQ, void *dK, void *dV,
                       int B, int H, int N, int D, int M, float eps, la_dtype t,
                       void *ws, size_t ws_bytes, void *stream);

/*
 * One recurrent decode step for B*H heads (eq. 16-20): update, then read.
 *   S <- S + phi(k) v^T,  z <- z + phi(k),  out = phi(q)^T S / (phi(q) . z + eps).
 * q, k [B,H,D] in; v [B,H,M] in; S [B,H,D,M] fp32 and z [B,H,D] fp32 in/out
 * (the caller zero-fills them before the first step, eq. 16-17, and may copy
 * them out and back to suspend and resume a sequence); out [B,H,M] out.
 * Successive steps on one stream are ordered by the stream.
 */
int la_recurrent_step(const void *q, const void *k, const void *v, float *S, float *z, void *out,
                      int B, int H, int D, int M, float eps, la_dtype t, void *stream);

/*
 * T consecutive decode steps in one launch (eq. 16-20 applied T times), for callers that
 * already hold every token's q, k, v (scoring a given sequence, teacher forcing): the state
 * stays on chip between steps, which removes the per-step launch that dominates the
 * single-step loop (the paper's "outer loop over the sequence", supplementary C).
 * q, k [T,B,H,D] in; v [T,B,H,M] in; out [T,B,H,M] out; S, z as in la_recurrent_step
 * (read at the start, written back at the end).  T >= 1.  Outputs and final state are
 * bit-identical to T calls of la_recurrent_step.
 */
int la_recurrent_steps(const void *q, const void *k, const void *v, float *S, float *z, void *out,
                       int T, int B, int H, int D, int M, float eps, la_dtype t, void *stream);

/*
 * Optional profiling hook (measurement aid, not part of the method).  The caller creates a
 * la_profile object and owns it.  Between la_profile_begin(p, mask) and la_profile_end(p, ...)
 * every launch that THE CALLING THREAD makes of a kernel whose bit (1u << la_kernel_id) is set
 * in `mask` is bracketed by two HIP events on the stream it is launched on.  la_profile_end
 * waits for those events, adds the elapsed milliseconds per kernel into ms_total[LA_K_COUNT]
 * and the number of launches into launches[LA_K_COUNT] (either may be NULL), and detaches the
 * object from the thread.  At most 8192 launches are recorded per window.  Nothing is shared
 * between threads or objects; an object must be used by one thread at a time.  begin / end
 * return LA_OK, LA_ERR_NULL or LA_ERR_HIP; la_profile_create returns NULL when out of memory.
 */
typedef struct la_profile la_profile;
typedef enum {
    LA_K_SEG_KV = 0,   /* per-segment sums of phi(K)^T V and phi(K)            */
    LA_K_SCAN = 1,     /* scan over the segment sums                           */
    LA_K_FWD = 2,      /* causal forward pass                                  */
    LA_K_GLOBAL = 3,   /* non-causal read-out                                  */
    LA_K_DQ = 4,       /* gradient for Q, 1/den, delta, per-segment Q,dO sums  */
    LA_K_REV = 5,      /* gradients for V and K (reverse direction)            */
    LA_K_STEP = 6,     /* recurrent decode step                                */
    LA_K_GLOBAL_BWD = 7, /* the non-causal read-outs for dV and dK, as one span */
    LA_K_COUNT = 8
} la_kernel_id;

const char *la_kernel_name(int kernel_id);
la_profile *la_profile_create(void);
void la_profile_destroy(la_profile *p);
int la_profile_begin(la_profile *p, unsigned mask);
int la_profile_end(la_profile *p, float *ms_total, int *launches);

#ifdef __cplusplus
}
#endif
#endif /* LA_H_ */
