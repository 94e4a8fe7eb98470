/*
 * flurka.h -- C ABI of the FLuRKA attention library for AMD MI355X (gfx950).
 *
 * FLuRKA (Fast Low-Rank & Kernel Attention) first contracts keys and values
 * along the sequence with two projection matrices, then applies a kernel
 * feature map and evaluates the attention product in the associative order
 * that never forms an n x k (or n x n) attention matrix:
 *
 *     K' = E K,  V' = F V                                  (n -> k rows)
 *     out = phi(Q) (phi(K')^T V')  /  phi(Q) (phi(K')^T 1)   (row-wise ratio)
 *
 * Source of each piece: the optimised unification, Eq. 2 (low-rank projection
 * before the kernel map); E, F in R^{k x n}, entries N(0, 1/k) -- Sec. 2,
 * "Low-rank Methods" (d_k and N there); phi and the product order
 * phi(Q)(phi(K)^T V) -- Sec. 2, "Kernel Methods"; the row normaliser -- the
 * ratio form used throughout App. D.  Eq. 2 is printed without the transpose
 * and the normaliser; both are meant.
 *
 * Feature maps:
 *   FLURKA_PHI_PERFORMER  positive random features,
 *                         phi(x)_j = exp(omega_j . x - |x|^2/2) / sqrt(m),
 *                         j = 1..m (Sec. 2: phi = m^{-1/2}[psi_1..psi_m] with
 *                         E[psi(x) psi(y)] = exp(x . y); Thm. 1 statement).
 *   FLURKA_PHI_ELU1       phi(x) = elu(x) + 1 elementwise, the non-random map
 *                         of the RNN variant (Sec. 2); then m must equal d and
 *                         omega is ignored (may be NULL).
 * The library applies no 1/sqrt(d) temperature, no mask, no dropout and adds
 * no epsilon to the denominator.  Exponents are shifted internally by one
 * constant per (batch, head, feature) on the key side, put back on the query
 * side, and by one constant per query row; all cancel exactly in the ratio.
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller.  The
 *     library allocates nothing, frees nothing and keeps no pointer after the
 *     call returns.  Tensors are dense, row-major, innermost index last.
 *   - Storage type `dtype` applies to Q, K, V, E, F, omega, out, dOut and all
 *     gradients.  `ctx` and `workspace` are always float32.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream); the call returns without synchronising.
 *   - Arguments are validated on the host before anything is launched; a
 *     failed validation launches nothing and touches no memory.
 *   - Calls that share a ctx or workspace buffer must be ordered on one stream.
 *   - Results are deterministic: no floating-point atomics are used.
 */
#ifndef FLURKA_H
#define FLURKA_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Entry points are the only symbols the shared library exports. */
#define FLURKA_API __attribute__((visibility("default")))

typedef enum {
    FLURKA_OK = 0,
    FLURKA_ERR_NULL = 1,         /* a required pointer is NULL */
    FLURKA_ERR_SHAPE = 2,        /* a dimension is < 1, too large, or m != d for ELU1 */
    FLURKA_ERR_DTYPE = 3,        /* unknown dtype / phi / algo value */
    FLURKA_ERR_UNSUPPORTED = 4,  /* valid problem the selected algo cannot run */
    FLURKA_ERR_WORKSPACE = 5,    /* ctx or workspace buffer too small */
    FLURKA_ERR_LAUNCH = 6,       /* the HIP runtime reported a launch error */
    FLURKA_ERR_ALIGN = 7         /* a pointer is not aligned to its element size (ctx/workspace: 256 B) */
} flurka_status;

typedef enum { FLURKA_F32 = 0, FLURKA_BF16 = 1 } flurka_dtype;
typedef enum { FLURKA_PHI_PERFORMER = 0, FLURKA_PHI_ELU1 = 1 } flurka_phi;

/* Kernel family.  AUTO picks the bf16 MFMA kernels when dtype and shape allow
 * (see flurka_fast_path_supported) and the generic fp32-arithmetic kernels
 * otherwise.  GENERIC forces the latter; FAST fails with
 * FLURKA_ERR_UNSUPPORTED instead of falling back. */
typedef enum { FLURKA_ALGO_AUTO = 0, FLURKA_ALGO_GENERIC = 1, FLURKA_ALGO_FAST = 2 } flurka_algo;

typedef enum { FLURKA_PASS_FWD = 0, FLURKA_PASS_BWD = 1 } flurka_pass;

/* Upper limits accepted by validation (host-checkable, no GPU needed). */
#define FLURKA_MAX_BATCH_HEADS 65535   /* B*H, one grid-z slot each */
#define FLURKA_MAX_FEATURE_DIM 4096    /* d, m */
#define FLURKA_MAX_SEQ (1 << 24)       /* n, k */

/* Library ABI version (major*100 + minor). */
FLURKA_API int flurka_version(void);

/* Human-readable name of a status code; never NULL. */
FLURKA_API const char* flurka_status_str(flurka_status s);

/* Bytes of the context buffer that carries state from the forward to the
 * backward pass: K', V' (B,H,k,d), S = phi(K')^T V' (B,H,mf,d),
 * z = phi(K')^T 1 (B,H,mf), the exponent shifts c (B,H,mf) and, per query row,
 * lse (B,H,n) = ln of the denominator phi(Q) z as the library scales it (below);
 * mf = m (performer) or d (elu1).  S and z are stored for phi(K') with column j
 * scaled by exp(-c_j) (c_j = max_r of the key exponent, 0 for elu1); the same
 * factor is put back on feature j of phi(Q), so the ratio is unchanged:
 * lse_i = ln sum_j exp(omega_j . q_i + c_j) z_j  (elu1: ln sum_j phi(q_i)_j z_j).
 * Returns 0 for an invalid shape. */
FLURKA_API size_t flurka_ctx_bytes(int B, int H, int n, int d, int k, int m,
                        flurka_dtype dtype, flurka_phi phi);

/* Offsets, in float32 elements from the start of ctx, of its six segments in
 * the order K', V', S, z, c, lse, written to the HOST array `offsets6`
 * (for inspection and tests).  Returns FLURKA_ERR_NULL / _SHAPE / _DTYPE on
 * bad arguments. */
FLURKA_API flurka_status flurka_ctx_layout(int B, int H, int n, int d, int k, int m,
                                flurka_dtype dtype, flurka_phi phi, size_t* offsets6);

/* Bytes of scratch the given pass needs for `algo` (AUTO = the maximum over
 * the paths AUTO may take).  Contents need not survive between calls.
 * Returns 0 for an invalid shape. */
FLURKA_API size_t flurka_workspace_bytes(int B, int H, int n, int d, int k, int m,
                              flurka_dtype dtype, flurka_phi phi,
                              flurka_pass pass, flurka_algo algo);

/* 1 if the bf16 MFMA kernels cover this problem for `pass`, else 0.  They take
 * bf16 storage, d = 64 or 128, n a multiple of 8 (forward) or of 32
 * (backward), any m and any
 * k, as long as the per-head operand images fit the 160 KiB of LDS of a
 * compute unit (random features, forward: m <= 512 at d = 64, m <= 288 at
 * d = 128; backward: m <= 288 at d = 64, m <= 256 at d = 128; ELU1: always). */
FLURKA_API int flurka_fast_path_supported(int B, int H, int n, int d, int k, int m,
                               flurka_dtype dtype, flurka_phi phi, flurka_pass pass);

/*
 * Forward: out = phi(Q)(phi(EK)^T FV) / phi(Q)(phi(EK)^T 1)   (Eq. 2 with the
 * App. D normaliser), per (batch, head).
 *
 *   Q, K, V   in   (B, H, n, d)
 *   E, F      in   (k, n)         one pair shared by every batch and head
 *   omega     in   (H, m, d) if omega_per_head != 0, else (m, d) shared by
 *                  all heads; ignored (may be NULL) for FLURKA_PHI_ELU1
 *   out       out  (B, H, n, d)   rounded once to `dtype` at the final store
 *   ctx       out  flurka_ctx_bytes(...) bytes, 256-byte aligned; holds the
 *                  key-side state and lse afterwards (input of flurka_attn_bwd)
 *   workspace      flurka_workspace_bytes(..., FLURKA_PASS_FWD, algo) bytes,
 *                  256-byte aligned scratch
 */
FLURKA_API flurka_status flurka_attn_fwd(const void* Q, const void* K, const void* V,
                              const void* E, const void* F, const void* omega,
                              void* out,
                              void* ctx, size_t ctx_bytes,
                              void* workspace, size_t workspace_bytes,
                              int B, int H, int n, int d, int k, int m,
                              int omega_per_head,
                              flurka_dtype dtype, flurka_phi phi, flurka_algo algo,
                              void* stream);

/*
 * flurka_attn_fwd for callers that cannot allocate device memory and have no scratch buffer of their
 * own to hand over: code running under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, results and error codes as flurka_attn_fwd, without `workspace`: the
 * scratch is a fixed array of FLURKA_STATIC_WORKSPACE_BYTES inside the library's device image (each
 * GPU the library runs on holds one copy until the process ends; its address is looked up on the first
 * call on a device).  The call allocates and frees nothing.  A problem whose forward workspace
 * (flurka_workspace_bytes(..., FLURKA_PASS_FWD, algo)) exceeds FLURKA_STATIC_WORKSPACE_BYTES is refused
 * with FLURKA_ERR_WORKSPACE before anything is launched.  Every call on a GPU uses that GPU's one
 * array: calls that overlap on one GPU (two streams, two threads) race, so order them on one stream.
 * The array keeps the previous call's contents; nothing in it has to start at zero (every kernel reads
 * only what an earlier kernel of the same call wrote).
 */
#define FLURKA_STATIC_WORKSPACE_BYTES (32u << 20)
FLURKA_API flurka_status flurka_attn_fwd_static(const void* Q, const void* K, const void* V,
                              const void* E, const void* F, const void* omega,
                              void* out,
                              void* ctx, size_t ctx_bytes,
                              int B, int H, int n, int d, int k, int m,
                              int omega_per_head,
                              flurka_dtype dtype, flurka_phi phi, flurka_algo algo,
                              void* stream);

/*
 * Forward with the linear transforms fused in the order Eq. 2 prints them:
 *
 *     K' = (E X_K) W^K_h,   V' = (F X_V) W^V_h,   out as in flurka_attn_fwd
 *
 * The sequence projection is applied once to the model-wide layer inputs X_K, X_V (before the split into
 * heads), and each head's transform to the k projected rows instead of the n sequence positions (App. B,
 * steps "downsampling" then "linear transformation": d_k d_m^2 instead of N d_m^2 products per
 * transform).  The result equals flurka_attn_fwd on K = X_K W^K_h, V = X_V W^V_h (the products
 * re-associate), up to rounding: here X W is never rounded to the storage type.
 *
 *   Q         in   (B, H, n, d)    per-head queries (already transformed)
 *   XK, XV    in   (B, n, dm)      layer inputs of the key and value branches, dm = model width
 *   WK, WV    in   (H, d, dm)      head h's transform stored transposed: row t holds column t of W_h
 *   E, F, omega, out, ctx           as in flurka_attn_fwd; ctx holds the same state afterwards
 *   workspace      flurka_fused_w_workspace_bytes(...) bytes, 256-byte aligned
 *
 * Only the bf16 MFMA kernels implement this order: bf16 storage, d = 64 or 128, n a multiple of 8, m within
 * the forward's limit, dm a multiple of 64, H*d a multiple of 256; anything else returns
 * FLURKA_ERR_UNSUPPORTED (flurka_fused_w_supported tells beforehand).  No backward pass is provided for
 * this entry point.
 */
FLURKA_API int flurka_fused_w_supported(int B, int H, int n, int d, int k, int m, int dm,
                             flurka_dtype dtype, flurka_phi phi);
FLURKA_API size_t flurka_fused_w_workspace_bytes(int B, int H, int n, int d, int k, int m, int dm,
                                      flurka_dtype dtype, flurka_phi phi);
FLURKA_API flurka_status flurka_attn_fwd_fused_w(const void* Q, const void* XK, const void* XV,
                              const void* E, const void* F, const void* WK, const void* WV,
                              const void* omega, void* out,
                              void* ctx, size_t ctx_bytes,
                              void* workspace, size_t workspace_bytes,
                              int B, int H, int n, int d, int k, int m, int dm,
                              int omega_per_head,
                              flurka_dtype dtype, flurka_phi phi,
                              void* stream);

/*
 * The method's two constituents as attention-level baselines, for the speed comparisons of Sec. 4.1
 * ("Model speed") and Sec. 4.3 (ablations over d_k and d_m) on this hardware.  Forward only, bf16 MFMA
 * kernels only (d = 64 or 128, n a multiple of 64); anything else returns FLURKA_ERR_UNSUPPORTED.
 *
 *   FLURKA_BASELINE_KERNEL_ATTN   kernel attention (Sec. 2, "Kernel Methods"):
 *                                 out = phi(Q)(phi(K)^T V) / phi(Q)(phi(K)^T 1), i.e. the forward above
 *                                 with E = F = I computed without any n x n product.  E, F and k are
 *                                 ignored (pass NULL, anything); m a multiple of 32.
 *   FLURKA_BASELINE_LINFORMER     low-rank attention (Sec. 2, "Low-rank Methods"):
 *                                 out = softmax(Q (E K)^T) (F V), softmax over the k projected keys, no
 *                                 temperature.  omega, m and phi are ignored.  The k projected keys and
 *                                 values of a head are kept in LDS as bf16: k <= 512 at d = 64,
 *                                 k <= 256 at d = 128 (rounded up to a multiple of 32).
 *
 * ctx (flurka_baseline_ctx_bytes) holds lse afterwards (and S, z, c resp. K', V'); workspace as
 * flurka_baseline_workspace_bytes says.  Conventions as for flurka_attn_fwd.
 */
typedef enum { FLURKA_BASELINE_KERNEL_ATTN = 0, FLURKA_BASELINE_LINFORMER = 1 } flurka_baseline;
FLURKA_API int flurka_baseline_supported(flurka_baseline which, int B, int H, int n, int d, int k, int m,
                              flurka_dtype dtype, flurka_phi phi);
FLURKA_API size_t flurka_baseline_ctx_bytes(flurka_baseline which, int B, int H, int n, int d, int k, int m,
                                 flurka_dtype dtype, flurka_phi phi);
FLURKA_API size_t flurka_baseline_workspace_bytes(flurka_baseline which, int B, int H, int n, int d, int k, int m,
                                       flurka_dtype dtype, flurka_phi phi);
FLURKA_API flurka_status flurka_baseline_fwd(flurka_baseline which,
                              const void* Q, const void* K, const void* V,
                              const void* E, const void* F, const void* omega,
                              void* out,
                              void* ctx, size_t ctx_bytes,
                              void* workspace, size_t workspace_bytes,
                              int B, int H, int n, int d, int k, int m,
                              int omega_per_head,
                              flurka_dtype dtype, flurka_phi phi,
                              void* stream);

/*
 * Backward of flurka_attn_fwd (chain rule; the paper trains through this
 * layer but prints no backward).  Given dOut = d loss / d out:
 *
 *   out         in   (B, H, n, d), the forward's result for the same inputs
 *                    (the row sums g_i of dOut * out enter every gradient; the
 *                    MFMA kernels take them from `out` as a first estimate and
 *                    correct it with their own attention weights, the generic
 *                    kernels recompute them and only check the pointer)
 *   dQ, dK, dV  out  (B, H, n, d)
 *   dE, dF      out  (k, n), summed over batch and heads (E, F are shared),
 *                    overwritten, not accumulated into
 *   ctx         in   the buffer filled by flurka_attn_fwd for the SAME
 *                    Q, K, V, E, F, omega and shape, earlier on this stream
 *
 * omega is a fixed random draw and gets no gradient.
 */
FLURKA_API flurka_status flurka_attn_bwd(const void* Q, const void* K, const void* V,
                              const void* E, const void* F, const void* omega,
                              const void* out, const void* dOut,
                              const void* ctx, size_t ctx_bytes,
                              void* dQ, void* dK, void* dV, void* dE, void* dF,
                              void* workspace, size_t workspace_bytes,
                              int B, int H, int n, int d, int k, int m,
                              int omega_per_head,
                              flurka_dtype dtype, flurka_phi phi, flurka_algo algo,
                              void* stream);

/*
 * Extended entry points: flurka_attn_fwd / flurka_attn_bwd with the variants of the method that the plain
 * ones leave out.  `options` == NULL, or all fields zero, is exactly the plain call (both kernel families).
 * Any option set runs on the generic (fp32-arithmetic) kernels: algo must be AUTO or GENERIC
 * (FAST returns FLURKA_ERR_UNSUPPORTED), and the workspace is the GENERIC one
 * (flurka_workspace_bytes(..., FLURKA_ALGO_GENERIC)).
 *
 *   ef_per_head   E, F are (H, k, n): one projection pair per head, as the statement of Thm. 1 writes them
 *                 (E_i, F_i); dE, dF are then (H, k, n) too, summed over the batch only.
 *   grad_ef_f32   backward: dE, dF are written as float32 whatever `dtype` is (they are sums over every
 *                 batch element, head and coordinate).
 *   d_omega       backward: if not NULL, receives d loss / d omega as float32, (H, m, d) or (m, d) like
 *                 omega itself (summed over the batch, and over the heads when omega is shared).  The
 *                 paper draws omega once and does not train it; this is for callers that do.  Must be
 *                 NULL for FLURKA_PHI_ELU1.
 * The forward uses ef_per_head only.
 */
typedef struct {
    int ef_per_head;
    int grad_ef_f32;
    void* d_omega;
} flurka_options;

FLURKA_API flurka_status flurka_attn_fwd_ex(const void* Q, const void* K, const void* V,
                              const void* E, const void* F, const void* omega,
                              void* out,
                              void* ctx, size_t ctx_bytes,
                              void* workspace, size_t workspace_bytes,
                              int B, int H, int n, int d, int k, int m,
                              int omega_per_head,
                              flurka_dtype dtype, flurka_phi phi, flurka_algo algo,
                              const flurka_options* options,
                              void* stream);
FLURKA_API flurka_status flurka_attn_bwd_ex(const void* Q, const void* K, const void* V,
                              const void* E, const void* F, const void* omega,
                              const void* out, const void* dOut,
                              const void* ctx, size_t ctx_bytes,
                              void* dQ, void* dK, void* dV, void* dE, void* dF,
                              void* workspace, size_t workspace_bytes,
                              int B, int H, int n, int d, int k, int m,
                              int omega_per_head,
                              flurka_dtype dtype, flurka_phi phi, flurka_algo algo,
                              const flurka_options* options,
                              void* stream);

/*
 * Built-in stage timer (for benchmarks; off by default, not thread-safe).
 * While enabled, every forward/backward call brackets each of its stages with
 * HIP events recorded on the call's own stream.  flurka_profile_read waits
 * for the recorded events, writes up to `capacity` (stage id, milliseconds)
 * pairs in launch order to the HOST arrays, forgets them and returns how many
 * it wrote (at most 4096 are kept between reads).  Enabling creates the
 * events (host-side resources only, no device memory); disabling destroys
 * them.  Stages: the sequence projections, the key-side state, the query
 * stream, and the backward stages (see flurka_profile_stage_name).
 */
FLURKA_API flurka_status flurka_profile_enable(int on);
FLURKA_API int flurka_profile_read(int* stage_ids, float* milliseconds, int capacity);
FLURKA_API const char* flurka_profile_stage_name(int stage_id);

#ifdef __cplusplus
}
#endif
#endif /* FLURKA_H */
