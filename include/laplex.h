/*
 * liblaplex — the LAPLEX apply on one MI355X (gfx950), C ABI.
 *
 *   y = L(a,b) x,   L_ij = exp(-|a_i - b_j|),   i < k outputs, j < n inputs
 *
 * (Introduction: the Laplace-kernel matrix; Sec. 3: the exact reduction of the
 * product to a sort and two decayed scans.)  Letters follow this library's
 * convention, not the theorems': `a` holds the k OUTPUT anchors, `b` the n
 * INPUT anchors, L is k x n.
 *
 * Common rules for every entry point
 *  - Every pointer is a DEVICE pointer unless marked "host".  The caller owns
 *    all buffers, including the workspace.  Inputs are const and untouched;
 *    outputs are overwritten, never accumulated into.
 *  - Batched data are batch-minor: element (row r, batch column t) of a matrix
 *    with leading dimension ld lives at [r*ld + t], ld >= batch.  batch == 1
 *    with ld == 1 is the plain-vector case.
 *  - Calls only enqueue work on `stream`; they never synchronise, allocate or
 *    free.  Two calls that share a workspace must be ordered by the caller
 *    (same stream, or events).
 *  - Return value: LAPLEX_OK or a negative LAPLEX_ERR_*.  Arguments are
 *    checked on the host before the first HIP call, so an argument error
 *    leaves every buffer untouched.  No exception crosses the boundary.
 *  - Limits: 0 <= k, n, batch; k + n <= LAPLEX_MAX_MERGED; float pointers
 *    4-byte aligned (16-byte aligned pointers with batch and ld multiples of 4
 *    take the 128-bit access path of the same kernels); `ws` 256-byte aligned.
 *  - Anchors must be finite.  NaN or infinite anchors give unspecified values
 *    but never a hang or an out-of-bounds access.  -0.0 is treated as +0.0.
 *  - Equal anchors are ordered "outputs by index, then inputs by index"
 *    (stable sort of a followed by b; Thm 1's half-open intervals put an input
 *    equal to an output after it).  The product does not depend on that order;
 *    anchor gradients use sgn(0) = 0 at ties, i.e. tied pairs contribute
 *    nothing to ga / gb (the paper prints no backward formula; this is the
 *    central-difference limit of the definition).
 *
 * Workspace.  laplex_workspace_bytes(k, n, batch, ...) gives the size for the
 * apply form; the Gram form of n anchors uses (k = 0, n, batch).  Its front
 * holds the PLAN of the anchors: the sorted order (ids) and the decay between
 * sorted neighbours.  The plan depends on the anchors only, so it stays valid
 * across batches and across the forward / backward pair until the anchors
 * change or the caller overwrites it (Sec. 3 "Complexity": the sorted order is
 * reused across batches).  After the plan comes the saved-scan region written
 * under LAPLEX_SAVE_SCANS, then scratch whose contents are undefined between
 * calls.
 *
 * Small problems.  With k + n <= 8192 the apply and Gram calls (and the calls
 * built on them) run in two launches: a sort by counting ranks over the whole
 * device and one kernel that holds the plan in LDS for the scans.  Arguments,
 * flags, workspace and results are the same (the sorted-input promises are then
 * not needed and not used); values differ from the large path's in rounding
 * only.
 */
#ifndef LAPLEX_H
#define LAPLEX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ihipStream_t* laplex_stream_t; /* a hipStream_t; NULL = the default stream */

enum {
    LAPLEX_OK = 0,
    LAPLEX_ERR_NULL = -1,      /* a required pointer is NULL */
    LAPLEX_ERR_SIZE = -2,      /* negative size, or k + n above LAPLEX_MAX_MERGED */
    LAPLEX_ERR_LD = -3,        /* a leading dimension below batch */
    LAPLEX_ERR_WORKSPACE = -4, /* ws_bytes below laplex_workspace_bytes(...) */
    LAPLEX_ERR_FLAGS = -5,     /* unknown bit, or a bit that has no meaning for this call */
    LAPLEX_ERR_HIP = -6,       /* a HIP launch failed; see laplex_last_hip_error() */
    LAPLEX_ERR_ALIGN = -7,     /* a float pointer not 4-byte, or ws not 256-byte, aligned */
    LAPLEX_ERR_VALUE = -8      /* a scalar argument is out of range (inverse temperature not positive and finite) */
};

enum {
    /* The caller promises a / b ascending.  With both set (or A_SORTED for the
     * Gram form) the radix sort is replaced by one merge-path pass.  A wrong
     * promise gives wrong values, never a fault. */
    LAPLEX_A_SORTED = 1u,
    LAPLEX_B_SORTED = 2u,
    /* The workspace already holds the plan of these same anchors (from an
     * earlier call with the same k, n, batch): skip sort, merge and decay. */
    LAPLEX_REUSE_PLAN = 4u,
    /* Forward calls: also store, per output row and batch column, the signed
     * difference of the strict right and left scans in the workspace.
     * Backward calls: that region was stored by the forward call on the same
     * (anchors, x); use it for the anchor gradient instead of re-scanning x. */
    LAPLEX_SAVE_SCANS = 8u
};

#define LAPLEX_MIX_MAX_OPERATORS 4096LL    /* operators summed by the laplex_mix_* calls */
#define LAPLEX_WGRAM_MAX_ANCHORS 1048576LL /* rows of the k x k weighted Gram matrix */
#define LAPLEX_MAX_MERGED 4294967294LL /* ids are 32-bit; 2^32-1 positions plus a sentinel slot */

/* Bytes of workspace for an apply with k outputs, n inputs and `batch`
 * columns (Gram form: k = 0).  `out` is a host pointer.  Pure host arithmetic. */
int laplex_workspace_bytes(int64_t k, int64_t n, int64_t batch, size_t* out);

/*
 * Forward apply (Sec. 3, Thm 1 / App. B "Matvec proofs"; computed here as one
 * sort of the merged anchors and a forward plus a backward decayed scan
 * s_j = exp(-(p_j - p_{j-1})) s_{j-1} + x_j over the merged sequence):
 *   y[i*ldy + t] = sum_j exp(-|a[i]-b[j]|) * x[j*ldx + t],   i<k, j<n, t<batch.
 * n == 0 writes zeros; k == 0 or batch == 0 does nothing.
 * Flags: A_SORTED, B_SORTED, REUSE_PLAN, SAVE_SCANS.
 */
int laplex_apply(const float* a, int64_t k, const float* b, int64_t n,
                 const float* x, int64_t ldx, int64_t batch,
                 float* y, int64_t ldy,
                 void* ws, size_t ws_bytes, uint32_t flags, laplex_stream_t stream);

/*
 * Backward of the apply for the loss sum_{i,t} gy[i*ldgy+t] * y[i*ldy+t]
 * (Sec. 5 / App. "Matvec benchmark": exact gradients w.r.t. x, a, b at the cost
 * of the forward's scans):
 *   gx[j*ldgx+t] = sum_i L_ij gy[i,t]
 *   ga[i] = -sum_t gy[i,t] sum_j sgn(a_i-b_j) L_ij x[j,t]
 *   gb[j] = +sum_t x[j,t]  sum_i sgn(a_i-b_j) L_ij gy[i,t]        (sgn(0) = 0)
 * Any of gx, ga, gb may be NULL (not wanted).  x may be NULL when both ga and
 * gb are NULL.  Empty sides give zeros in whatever is wanted.
 * Flags: A_SORTED, B_SORTED, REUSE_PLAN, SAVE_SCANS (see above).
 */
int laplex_apply_backward(const float* a, int64_t k, const float* b, int64_t n,
                          const float* x, int64_t ldx,
                          const float* gy, int64_t ldgy, int64_t batch,
                          float* gx, int64_t ldgx, float* ga, float* gb,
                          void* ws, size_t ws_bytes, uint32_t flags, laplex_stream_t stream);

/*
 * For callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  The forward apply with
 * its workspace inside the library: a file-scope device array of
 * LAPLEX_STATIC_WORKSPACE_BYTES that every GPU the library runs on holds until
 * the process ends.  Same arguments, layout, limits and results (bit for bit) as
 * laplex_apply without `ws`; flags: A_SORTED, B_SORTED only (there is no plan or
 * saved scan to hand to a later call: LAPLEX_ERR_FLAGS).  Problems whose
 * laplex_workspace_bytes(k, n, batch) exceeds LAPLEX_STATIC_WORKSPACE_BYTES are
 * rejected with LAPLEX_ERR_WORKSPACE before anything is enqueued.  The call
 * allocates and frees nothing; it works on the device that is current when it is
 * called, which must be the device of `stream`.  The first call on a device looks
 * the array's address up (no allocation; make that call outside graph capture).
 * All calls on one device share that device's array: calls that may overlap on
 * one device (different streams, or threads) race and must be ordered by the
 * caller.  Nothing in the array has to survive from one call to the next; every
 * call rebuilds what it reads.
 */
#define LAPLEX_STATIC_WORKSPACE_BYTES 33554432ULL /* 32 MiB */

int laplex_apply_static(const float* a, int64_t k, const float* b, int64_t n,
                        const float* x, int64_t ldx, int64_t batch,
                        float* y, int64_t ldy, uint32_t flags, laplex_stream_t stream);

/*
 * Square (Gram) form K = L(a,a) (Sec. 3 "Symmetric case": sorted a, a prefix
 * and a suffix scan):  y[m*ldy+t] = sum_j exp(-|a[m]-a[j]|) x[j*ldx+t].
 * Flags: A_SORTED, REUSE_PLAN, SAVE_SCANS.
 */
int laplex_gram(const float* a, int64_t n, const float* x, int64_t ldx, int64_t batch,
                float* y, int64_t ldy,
                void* ws, size_t ws_bytes, uint32_t flags, laplex_stream_t stream);

/*
 * Backward of the Gram form for the loss sum gy.y:
 *   gx = K gy,
 *   ga[m] = sum_t [ gy[m,t] sum_j s_mj K_mj x[j,t] + x[m,t] sum_i s_mi K_im gy[i,t] ],
 *   s_mj = -sgn(a_m - a_j)   (duplicates and the diagonal contribute 0).
 * gx or ga may be NULL.  Flags: A_SORTED, REUSE_PLAN, SAVE_SCANS.
 */
int laplex_gram_backward(const float* a, int64_t n, const float* x, int64_t ldx,
                         const float* gy, int64_t ldgy, int64_t batch,
                         float* gx, int64_t ldgx, float* ga,
                         void* ws, size_t ws_bytes, uint32_t flags, laplex_stream_t stream);

/*
 * Temperature (App. A, "Expressivity": the temperature-scaled kernel
 * exp(-|a_i - b_j| / t); the experiments' inverse temperature tau = 1/t):
 *
 *   L_tau = [exp(-tau * |a_i - b_j|)],   tau > 0 and finite (host scalar)
 *
 * The four calls below are the four above on the anchors tau*a, tau*b, scaled
 * in fp32 on the way into the sort (the sorted order and the tie rule are those
 * of the scaled anchors); a plan is valid for the tau it was built with.
 * Gradients are with respect to the caller's a, b; gtau (device, one float,
 * may be NULL) receives d/d tau = sum_i a_i ga_i/tau + sum_j b_j gb_j/tau, in a
 * fixed summation order; it is formed from ga and gb, which must then both be
 * given (ga for the Gram form).  tau == 1 gives the bits of the plain calls.
 */
int laplex_apply_tau(const float* a, int64_t k, const float* b, int64_t n, float tau,
                     const float* x, int64_t ldx, int64_t batch, float* y, int64_t ldy,
                     void* ws, size_t ws_bytes, uint32_t flags, laplex_stream_t stream);
int laplex_apply_backward_tau(const float* a, int64_t k, const float* b, int64_t n, float tau,
                              const float* x, int64_t ldx, const float* gy, int64_t ldgy, int64_t batch,
                              float* gx, int64_t ldgx, float* ga, float* gb, float* gtau,
                              void* ws, size_t ws_bytes, uint32_t flags, laplex_stream_t stream);
int laplex_gram_tau(const float* a, int64_t n, float tau, const float* x, int64_t ldx, int64_t batch,
                    float* y, int64_t ldy, void* ws, size_t ws_bytes, uint32_t flags, laplex_stream_t stream);
int laplex_gram_backward_tau(const float* a, int64_t n, float tau, const float* x, int64_t ldx,
                             const float* gy, int64_t ldgy, int64_t batch, float* gx, int64_t ldgx,
                             float* ga, float* gtau,
                             void* ws, size_t ws_bytes, uint32_t flags, laplex_stream_t stream);

/*
 * Phased kernel (Sec. 3, "Phased Laplace kernels"):
 *
 *   y[i*ldy + t] = sum_j exp(-|a[i] - b[j]|) * cos(phi[i] - psi[j]) * x[j*ldx + t]
 *
 * phi[k] are the phases of the output anchors, psi[n] those of the input
 * anchors (radians).  By the angle-sum identity the product is two plain
 * products on a doubled batch plus pointwise modulation, which is how it is
 * computed: the workspace (laplex_phased_workspace_bytes) holds the plain
 * workspace for batch 2*batch at its front (the plan, as above) and the cosine
 * and sine halves of x, y, gy and gx behind it.  Same flags as laplex_apply;
 * LAPLEX_SAVE_SCANS also keeps the halves of x and of the product for
 * laplex_phased_apply_backward.  Limits as above with 2*batch for batch.
 */
int laplex_phased_workspace_bytes(int64_t k, int64_t n, int64_t batch, size_t* out /* host */);

int laplex_phased_apply(const float* a, const float* phi, int64_t k,
                        const float* b, const float* psi, int64_t n,
                        const float* x, int64_t ldx, int64_t batch, float* y, int64_t ldy,
                        void* ws, size_t ws_bytes, uint32_t flags, laplex_stream_t stream);

/*
 * Gradients of sum(gy * y) of the phased product: gx[n][batch], ga[k], gb[n],
 * gphi[k], gpsi[n]; any of them may be NULL (= not wanted).  x may be NULL if
 * only gx is wanted.  Anchor gradients follow the tie rule above (tied pairs
 * contribute nothing); the phase gradients are
 *   gphi[i] = -sum_t gy[i,t] sum_j exp(-|a_i - b_j|) sin(phi_i - psi_j) x[j,t]
 *   gpsi[j] = +sum_t x[j,t]  sum_i exp(-|a_i - b_j|) sin(phi_i - psi_j) gy[i,t].
 * With LAPLEX_SAVE_SCANS (and LAPLEX_REUSE_PLAN) the call continues a
 * laplex_phased_apply on the same anchors, phases, x and workspace; without,
 * it stands alone (and, if gphi is wanted, computes the forward product itself).
 */
int laplex_phased_apply_backward(const float* a, const float* phi, int64_t k,
                                 const float* b, const float* psi, int64_t n,
                                 const float* x, int64_t ldx, const float* gy, int64_t ldgy, int64_t batch,
                                 float* gx, int64_t ldgx, float* ga, float* gb, float* gphi, float* gpsi,
                                 void* ws, size_t ws_bytes, uint32_t flags, laplex_stream_t stream);

/*
 * LAPLEX^(r): a weighted sum of r operators with independent anchor pairs
 * (Sec. 7, "Learned anchor geometry in neural heads"):
 *
 *   y[i*ldy + t] = sum_q w[q] * sum_j exp(-|a[q*k + i] - b[q*n + j]|) * x[j*ldx + t]
 *
 * a[r][k], b[r][n] contiguous, w[r] in DEVICE memory (the mixing weights are
 * trained like the anchors), r <= LAPLEX_MIX_MAX_OPERATORS.  Computed as r plain
 * applies whose products are combined in a fixed order.  The workspace
 * (laplex_mix_workspace_bytes) holds r plain workspaces back to back (operator q's
 * plan sits at q * (their common size); the flags act on every operator alike),
 * then the r products and the scratch of the backward call.
 * laplex_mix_apply_backward: gradients of sum(gy * y): gx[n][batch], ga[r][k],
 * gb[r][n] (tie rule as above), gw[r] = <gy, L_q x>; any may be NULL.  With
 * LAPLEX_SAVE_SCANS the forward call (same flag, same workspace) has left what the
 * backward needs; without it the products needed for gw are recomputed.  x may be
 * NULL if only gx is wanted.  r == 0 gives y = 0.
 * Streams: everything is ordered after the work already in `stream`, and work put
 * into `stream` afterwards is ordered after everything these calls do.  In between,
 * operators with more than 8192 merged positions and small matrices may run on up to
 * four streams that the library creates once per device (default priority) and keeps;
 * while `stream` is being captured into a graph they stay on it.  The results do not
 * depend on which of the two happens.  Calls on different host threads take turns
 * while they enqueue.
 */
int laplex_mix_workspace_bytes(int64_t r, int64_t k, int64_t n, int64_t batch, size_t* out /* host */);

int laplex_mix_apply(const float* a, const float* b, const float* w, int64_t r, int64_t k, int64_t n,
                     const float* x, int64_t ldx, int64_t batch, float* y, int64_t ldy,
                     void* ws, size_t ws_bytes, uint32_t flags, laplex_stream_t stream);

int laplex_mix_apply_backward(const float* a, const float* b, const float* w, int64_t r, int64_t k, int64_t n,
                              const float* x, int64_t ldx, const float* gy, int64_t ldgy, int64_t batch,
                              float* gx, int64_t ldgx, float* ga, float* gb, float* gw,
                              void* ws, size_t ws_bytes, uint32_t flags, laplex_stream_t stream);

/*
 * Weighted Gram matrix (Sec. 3, "Computation of Gram matrix"; App. "Fast weighted
 * Gram matrix", Thm "Exact Gram decomposition"):
 *
 *   m[i*ldm + j] = sum_t d[t] * exp(-|a[i] - b[t]|) * exp(-|a[j] - b[t]|),   i, j < k, t < n
 *
 * i.e. M = A diag(d) A^T with A = L(a, b): a[k] are the anchors of the k x k
 * result, b[n] the middle anchors that are summed over, d[n] their weights (any
 * sign).  Cost O(k^2 + n log n): one sort of the doubled anchors, one forward and
 * one backward decayed scan of d, one fp64 prefix sum of d, then the k x k fill;
 * the full matrix is written (both triangles), rows ldm >= k floats apart.
 * k <= LAPLEX_WGRAM_MAX_ANCHORS.  Flags: LAPLEX_A_SORTED | LAPLEX_B_SORTED (both
 * set: merge instead of sort), LAPLEX_REUSE_PLAN (the workspace holds the plan of
 * an earlier laplex_wgram call with the same a, b).  n == 0 gives M = 0.  The
 * workspace is laplex_wgram_workspace_bytes(k, n); its front is a plan of the
 * anchors 2a, 2b (laplex_get_perm reads it): anchors beyond 1.7e38 in magnitude
 * overflow when doubled and are unsupported like infinite ones.  No gradients
 * are provided.
 */
int laplex_wgram_workspace_bytes(int64_t k, int64_t n, size_t* out /* host */);

int laplex_wgram(const float* a, int64_t k, const float* b, int64_t n, const float* d,
                 float* m, int64_t ldm, void* ws, size_t ws_bytes, uint32_t flags, laplex_stream_t stream);

/*
 * The weighted Gram matrix in fp64 (App. "Density model": the Gram matrices run in
 * fp64 through the same scan): fp32 anchors a[k], b[n]; fp64 weights d[n] and fp64
 * result m (k x k, rows ldm doubles apart; d and m 8-byte aligned).  The sorted
 * order and the ties are those of the fp32 anchors; every decay, product and sum is
 * formed in fp64.  Same flags, limits and plan as laplex_wgram; the workspace is
 * laplex_wgram_f64_workspace_bytes(k, n).
 */
int laplex_wgram_f64_workspace_bytes(int64_t k, int64_t n, size_t* out /* host */);

int laplex_wgram_f64(const float* a, int64_t k, const float* b, int64_t n, const double* d,
                     double* m, int64_t ldm, void* ws, size_t ws_bytes, uint32_t flags, laplex_stream_t stream);

/*
 * Verification hook: copy the first `count` sorted ids of the plan in `ws`
 * (count = k + n for the apply form, n for the Gram form) to the device buffer
 * perm_out.  id < k names output anchor a[id]; id >= k names input b[id-k].
 */
int laplex_get_perm(const void* ws, size_t ws_bytes, int64_t count, uint32_t* perm_out,
                    laplex_stream_t stream);

/*
 * An invalid plan is never silent.  The radix sort's tiles wait for their
 * predecessors' digit counts with a bounded spin, so that a lost wake-up can
 * never hang the device; a tile that gives up marks the plan invalid.  Every
 * call that computes from an invalid plan (the call that built it and every
 * later LAPLEX_REUSE_PLAN call on the same workspace) still returns LAPLEX_OK,
 * since nothing synchronises, but writes NaN to every element of every output
 * it produces (y, gx, ga, gb, gtau, the weighted Gram matrix, the products and
 * gradients of the phased and mixed calls): the kernels that store results read
 * the plan's status word and set every exponent and a mantissa bit of what they
 * store.  Repeating the call without LAPLEX_REUSE_PLAN rebuilds the plan.
 * Plans of at most 8192 positions and merged plans (both inputs promised
 * sorted) never wait and are always valid.
 *
 * laplex_get_plan_status writes the status word of the plan in `ws` (count =
 * k + n for the apply form, n for the Gram form) to the device word
 * status_out: 0 = valid, 1 = invalid.
 */
int laplex_get_plan_status(const void* ws, size_t ws_bytes, int64_t count, uint32_t* status_out,
                           laplex_stream_t stream);

/* Host: static text for a status code. */
const char* laplex_status_string(int status);

/* Host: text of the last HIP error this thread's calls ran into ("" if none). */
const char* laplex_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* LAPLEX_H */
