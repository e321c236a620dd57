/*
 * stl.h -- C ABI of the Strassen-Tile (STL) operator library for AMD MI355X (gfx950).
 *
 * The operator (paper: Definition 3.1, Eq. (2)) replaces C = X*W by
 *
 *     vec(C_{I,J}) = D^T ( sum_L (E_X vec X_{I,L}) (.) What[:,L,J] ),     t x t tiles,
 *
 * evaluated with the three-step plane algorithm (Claim 3.4, Algorithm 1):
 * (i) encode X tiles into r planes, (ii) r independent plane products on the matrix
 * cores, (iii) decode every output tile once.  What are the stored encoded weight
 * planes (Remark "Fake Encoding"): What[p][L][J] = (E_W vec W_{L,J})_p.
 *
 * Letters: X is m x k, W is k x n, C is m x n; M=m/t, K=k/t, N=n/t tile counts.
 *
 * Conventions for every entry point
 *  - All matrices are dense, row-major, without strides.  vec() of a tile is
 *    row-major: vec(T)[a*t+b] = T[a][b].  E_X, E_W, D are r x t^2 row-major
 *    (Definition 3.1); the decoder is applied as D^T.
 *  - Weight-side plane tensors (What, dWhat) are plane-major: [p][row tile][col tile].
 *  - Activation-side plane tensors (Xhat, Yhat; the library's dYhat and dXhat scratch alike) are plane-major
 *    within groups of STL_PLANE_GROUP = 64 tile rows: element (p, I, J) of an r x R x Cc tensor lives at
 *        ((I / 64) * r + p) * 64 * Cc + (I % 64) * Cc + J,
 *    and a buffer holds stl_plane_elems(R, Cc, r) = r * roundup(R, 64) * Cc elements.  (The r segments of
 *    one tile row then lie within r * 64 * Cc elements of each other instead of a whole plane apart, which
 *    the encode / decode passes need for speed, while 64 consecutive rows of a plane stay contiguous for
 *    the plane products.)  Callers that only pass Xhat_save / Yhat_save from stl_forward to stl_backward
 *    never need to know.
 *  - Every data pointer is a DEVICE pointer owned by the caller, 16-byte aligned
 *    (STL_ERR_INVALID_ARG otherwise).
 *    The library allocates and frees no device memory: scratch comes from `ws`
 *    (size from stl_workspace_bytes).  Outputs must not alias inputs or `ws`.
 *  - Calls only enqueue work on `stream` (a hipStream_t passed as void*; NULL is
 *    the default stream); they never synchronise and keep no state between calls.
 *  - Every argument is validated before any launch.  Nothing is launched when a
 *    non-STL_OK status is returned for an argument error.  Supported: t == 4,
 *    1 <= r <= 64, m, k, n positive multiples of t not above STL_MAX_DIM, dtype in {F32, BF16}.
 *  - dtype selects the storage type of X, W, What, E_X, E_W, D, C, dC, dX, Xhat,
 *    Yhat.  Arithmetic: fp32 multiply-add throughout for F32; for BF16 the plane
 *    products are bf16 x bf16 -> fp32 on MFMA, encode/decode are fp32, and each
 *    stored intermediate (Xhat, Yhat when it leaves registers, dYhat, dXhat) and
 *    each output is rounded to bf16 once (round-to-nearest-even).
 *    dWhat, dE_X, dD are always fp32.
 *  - No exception or abort crosses this boundary.
 */
#ifndef STL_H_
#define STL_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    STL_OK = 0,
    STL_ERR_INVALID_ARG = 1,   /* null pointer, non-positive or non-divisible size, r out of range */
    STL_ERR_UNSUPPORTED = 2,   /* t != 4, unknown dtype or flag */
    STL_ERR_WORKSPACE = 3,     /* ws is NULL or ws_bytes too small */
    STL_ERR_HIP = 4            /* a HIP call failed; text in stl_last_error() */
} stl_status_t;

typedef enum { STL_F32 = 0, STL_BF16 = 1 } stl_dtype_t;

typedef struct {
    int64_t m, k, n;   /* X is m x k, What encodes a k x n weight, C is m x n */
    int32_t t, r;      /* tile size (4) and tensor rank (number of planes) */
    int32_t dtype;     /* stl_dtype_t */
} stl_problem_t;

/* Largest m, k or n (and largest stacked row count of the batched entry points): 65535 * 256, so that every launch
 * extent of every kernel, the any-shape ones included, stays within the device's grid limits. */
#define STL_MAX_DIM 16776960
#define STL_PLANE_GROUP 64
/* Elements of an activation-side plane tensor with r planes of R x Cc tiles (rows rounded up to the group). */
size_t stl_plane_elems(int64_t R, int64_t Cc, int r);

/* which operation a workspace is sized for */
enum { STL_OP_ENCODE_WEIGHT = 0, STL_OP_FORWARD = 1, STL_OP_BACKWARD = 2, STL_OP_ENCODE_WEIGHT_BACKWARD = 3 };

/* forward variants (low byte of `flags`) and modifiers */
enum {
    STL_FLAG_AUTO = 0,      /* library picks the fastest variant for the shape */
    STL_FLAG_UNFUSED = 1,   /* Algorithm 1 as three launches: encode -> plane products -> decode   */
    STL_FLAG_EPILOGUE = 2,  /* encode launch, then plane products with D applied in the epilogue   */
    STL_FLAG_FUSED = 3,     /* one launch: encode -> MFMA -> decode, no plane ever written to HBM   */
    STL_FLAG_PIPELINED = 4, /* one persistent launch over the three-launch kernels' own code: encode and decode items of
                               neighbouring row blocks run on some CUs while others multiply; same planes in HBM and
                               bit-identical results; bf16, r <= 32, k and n multiples of 256, n >= 1024,
                               2048 <= m <= 4194304 (else UNSUPPORTED) */
    STL_FLAG_VARIANT_MASK = 0xff,
    STL_FLAG_GELU = 0x100,  /* C <- gelu(C) (exact erf form) applied in fp32 before the final rounding */
    STL_FLAG_B_TRANSPOSED = 0x200   /* stl_aa_*: the second operand is stored transposed, (nbatch*n) x k */
};

/* Bytes of device scratch `ws` needed by op (STL_OP_*) with `flags`; 0 on invalid problem. */
size_t stl_workspace_bytes(const stl_problem_t *prob, int op, int flags);

/*
 * W-encoding (plane definition before Claim 3.4; Remark "Fake Encoding"):
 *   What[p][L][J] = sum_q E_W[p][q] * vec(W_{L,J})[q].
 * W: k x n (in).  E_W: r x 16 (in).  What: r x K x N (out).  Set-up cost, off the hot path.
 */
stl_status_t stl_encode_weight(const stl_problem_t *prob, const void *W, const void *E_W,
                               void *What, void *stream);

/*
 * Gradients through the W-encoding, for training W and E_W themselves instead of the encoded planes
 * (Section "Strassen-Tile Operator": gradients are taken with respect to E_X, E_W, D and W):
 *   dw[L][J][q] = sum_p E_W[p][q] dWhat[p][L][J]   -> dW,      dE_W[p][q] = sum_{L,J} dWhat[p][L][J] w[L][J][q].
 * W: k x n, E_W: r x 16 (in).  dWhat: r x K x N fp32 (in), as written by stl_backward.
 * dW: k x n (out, storage dtype) or NULL.  dE_W: r x 16 fp32 (out) or NULL; accumulate as in stl_backward
 * (applies to dE_W).  For BF16 storage dWhat is rounded to bf16 once before both sums.
 * ws / ws_bytes: at least stl_workspace_bytes(prob, STL_OP_ENCODE_WEIGHT_BACKWARD, 0).
 */
stl_status_t stl_encode_weight_backward(const stl_problem_t *prob, const void *W, const void *E_W,
                                        const float *dWhat, void *dW, float *dE_W, int accumulate,
                                        void *ws, size_t ws_bytes, void *stream);

/*
 * Forward C = X <> W (Definition 3.1 / Eq. (2); Algorithm 1).
 * X: m x k (in).  What: r x K x N (in).  E_X, D: r x 16 (in).  C: m x n (out).
 * Xhat_save: NULL, or stl_plane_elems(M, K, r) elements (out, storage dtype, grouped layout): the encoded activations of step (i) are
 *   written there instead of into the workspace, for stl_backward.
 * Yhat_save: NULL, or stl_plane_elems(M, N, r) elements (out, storage dtype, grouped layout): the encoded output
 *   Yhat[p] = Xhat[p] * What[p] (Claim 3.4) is also written there, for stl_backward.
 * ws / ws_bytes: scratch of at least stl_workspace_bytes(prob, STL_OP_FORWARD, flags).
 */
stl_status_t stl_forward(const stl_problem_t *prob, const void *X, const void *What,
                         const void *E_X, const void *D, void *C, void *Xhat_save, void *Yhat_save,
                         void *ws, size_t ws_bytes, int flags, void *stream);

/*
 * stl_forward for callers that cannot allocate device memory and have no workspace to pass: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same operator, same kernels and same results as
 * stl_forward(..., Xhat_save = NULL, Yhat_save = NULL, flags = STL_FLAG_UNFUSED | (flags & STL_FLAG_GELU)) taken in
 * one slab, but the two plane tensors (Xhat, Yhat) live in a scratch array built into the library's device code
 * (STL_STATIC_SCRATCH_BYTES per GPU, held from the library's first use on that GPU until the process ends) instead
 * of a caller workspace.  The call itself allocates and frees nothing.
 * X, What, E_X, D (in), C (out): as for stl_forward.  flags: 0 or STL_FLAG_GELU (anything else: STL_ERR_UNSUPPORTED).
 * Limit: stl_workspace_bytes(prob, STL_OP_FORWARD, STL_FLAG_UNFUSED) must not exceed STL_STATIC_SCRATCH_BYTES, i.e.
 *   r * roundup(M, 64) * (K + N) * sizeof(element), each tensor rounded up to 256 bytes; larger problems are rejected
 *   with STL_ERR_WORKSPACE before anything is launched.
 * The first call on a device looks up that device's copy of the array (hipGetSymbolAddress); make that call outside
 * a graph capture.  All calls on one GPU share the one array, which keeps the previous call's contents (every element
 * a call reads it has written before): calls that overlap in time on one GPU -- on different streams or from different
 * threads -- race; calls on one stream are ordered by the stream.
 */
#define STL_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
stl_status_t stl_forward_static(const stl_problem_t *prob, const void *X, const void *What,
                                const void *E_X, const void *D, void *C, int flags, void *stream);

/*
 * Backward of the scalar <dC, C> (chain rule through Algorithm 1's three linear steps;
 * the paper states only that these gradients exist, Section "Strassen-Tile Operator"):
 *   dYhat[p][I][J] = sum_q D[p][q] dc[I][J][q]          dD[p][q]   = sum_{I,J} Yhat[p][I][J] dc[I][J][q]
 *   dXhat[p] = dYhat[p] * What[p]^T                     dWhat[p]   = Xhat[p]^T * dYhat[p]
 *   dx[I][L][q] = sum_p E_X[p][q] dXhat[p][I][L]        dE_X[p][q] = sum_{I,L} dXhat[p][I][L] x[I][L][q]
 * dC: m x n (in).  Xhat_saved / Yhat_saved: NULL (recomputed here) or what stl_forward wrote to
 *   Xhat_save / Yhat_save for the same X, What, E_X.
 * dX: m x k (out, storage dtype).  dWhat: r x K x N, dE_X, dD: r x 16 (out, fp32).
 * Any of the four outputs may be NULL to skip it.
 * accumulate: 0 overwrites dWhat/dE_X/dD; 1 adds into them (fp32 gradient accumulation).
 * Results are bitwise reproducible run to run (no floating-point atomics).
 */
stl_status_t stl_backward(const stl_problem_t *prob, const void *X, const void *What,
                          const void *E_X, const void *D, const void *dC, const void *Xhat_saved,
                          const void *Yhat_saved, void *dX, float *dWhat, float *dE_X, float *dD, int accumulate,
                          void *ws, size_t ws_bytes, void *stream);

/*
 * The three steps of Algorithm 1 on their own (for measurement and stage-level tests).
 *   stl_encode_activation: Xhat[p][I][L] = (E_X vec X_{I,L})_p        X m x k -> Xhat r x M x K
 *   stl_plane_matmul:      Yhat[p] = Xhat[p] * What[p]  (Claim 3.4)    -> Yhat r x M x N
 *   stl_decode:            vec(C_{I,J}) = D^T Yhat[:,I,J]              -> C m x n   (flags: STL_FLAG_GELU or 0)
 */
stl_status_t stl_encode_activation(const stl_problem_t *prob, const void *X, const void *E_X,
                                   void *Xhat, void *stream);
stl_status_t stl_plane_matmul(const stl_problem_t *prob, const void *Xhat, const void *What,
                              void *Yhat, void *stream);
stl_status_t stl_decode(const stl_problem_t *prob, const void *Yhat, const void *D, void *C,
                        int flags, void *stream);

/*
 * Two stacked STL layers, C = (act(X <> W1)) <> W2 (Algorithm 2; Section "Strassen-Tile Operator",
 * paragraph on fusing step (iii) of one layer with step (i) of the next).  `up` describes the first
 * layer (X m x k1 -> n1), `down` the second (m x k2 -> n2) with down.m == up.m, down.k == up.n, same t
 * and dtype; the ranks may differ.  Output tile (I,J) of the first layer is input tile (I,L=J) of the
 * second, so decode, activation and the next encode are done per tile in one pass over the planes and
 * the hidden activation (m x n1) is never written:
 *     Xhat2[s][I][J] = sum_q E_X2[s][q] act( sum_p D1[p][q] Yhat1[p][I][J] ).
 * flags: STL_FLAG_GELU applies the exact-erf GELU between the layers (evaluated in fp32, rounded to
 *   the storage dtype before the second encode); without it the step is the paper's linear map
 *   Yhat1 (D1 E_X2^T) per tile.  Variant STL_FLAG_AUTO uses the one-pass step where its kernel
 *   applies (bf16, n1/4 a multiple of 8); STL_FLAG_UNFUSED always runs decode and encode as two
 *   launches through a hidden-activation buffer in the workspace.  Other variant values: UNSUPPORTED.
 * X: m x k1 (in).  What1: r1 x K1 x N1, What2: r2 x N1 x N2 (in).  E_X1, D1: r1 x 16; E_X2, D2: r2 x 16 (in).
 * C: m x n2 (out).  ws / ws_bytes: at least stl_mlp_workspace_bytes(up, down, flags).
 */
size_t stl_mlp_workspace_bytes(const stl_problem_t *up, const stl_problem_t *down, int flags);
stl_status_t stl_mlp_forward(const stl_problem_t *up, const stl_problem_t *down, const void *X,
                             const void *What1, const void *E_X1, const void *D1, const void *What2,
                             const void *E_X2, const void *D2, void *C, void *ws, size_t ws_bytes,
                             int flags, void *stream);
/*
 * The inter-layer step of stl_mlp_forward on its own: Yhat1 r1 x M x N1 (in), D1 r1 x 16, E_X2 r2 x 16
 * (in) -> Xhat2 r2 x M x N1 (out).  H: scratch for the hidden activation, m x n1 elements of the storage
 * dtype; may be NULL when the one-pass kernel applies (bf16 and n1/4 a multiple of 8) and the variant is
 * STL_FLAG_AUTO, required otherwise (INVALID_ARG if missing).  flags as for stl_mlp_forward.
 */
stl_status_t stl_recode(const stl_problem_t *up, const stl_problem_t *down, const void *Yhat1,
                        const void *D1, const void *E_X2, void *Xhat2, void *H, int flags, void *stream);

/*
 * STL of two activations, C_b = A_b <> B_b for b < nbatch (the attention products Q K^T and A V of the
 * Class-1 discussion: "activation x activation", where neither operand is a stored weight).  The second
 * operand is encoded at run time with E_B exactly as a weight is with E_W (plane definition before Claim
 * 3.4), the first with E_A as an activation:
 *     vec(C_b{I,J}) = D^T sum_L (E_A vec A_b{I,L}) (.) (E_B vec B_b{L,J}).
 * The nbatch independent problems (heads x images) are stacked along the rows and share the bases:
 * A: (nbatch*m) x k, B: (nbatch*k) x n, C: (nbatch*m) x n, prob giving m, k, n of ONE problem.
 * All plane tensors are activation-side (grouped layout) over the stacked tile rows:
 *   Ahat stl_plane_elems(nbatch*M, K, r), Bhat stl_plane_elems(nbatch*K, N, r), Yhat stl_plane_elems(nbatch*M, N, r)
 * elements.  *_save: NULL or a buffer that receives the tensor for stl_aa_backward.
 * flags: any of STL_FLAG_GELU and STL_FLAG_B_TRANSPOSED.  With STL_FLAG_B_TRANSPOSED the second operand is given
 * as its transpose, B: (nbatch*n) x k (Q K^T with K stored tokens x width), and the operator is applied to B_b^T: a tile
 * of B^T is the transpose of a tile of B, so B is encoded as it lies with the columns of E_B permuted accordingly, and the
 * planes are held as [p][J][L]: Bhat_save then has stl_plane_elems(nbatch*N, K, r) elements, and dB has B's shape.
 * ws / ws_bytes: at least stl_aa_workspace_bytes(prob, nbatch, STL_OP_FORWARD).
 * nbatch*m, nbatch*k and nbatch*n may not exceed STL_MAX_DIM (INVALID_ARG).  The workspace size does not depend on the flags.
 */
size_t stl_aa_workspace_bytes(const stl_problem_t *prob, int64_t nbatch, int op);
stl_status_t stl_aa_forward(const stl_problem_t *prob, int64_t nbatch, const void *A, const void *B,
                            const void *E_A, const void *E_B, const void *D, void *C, void *Ahat_save,
                            void *Bhat_save, void *Yhat_save, void *ws, size_t ws_bytes, int flags,
                            void *stream);
/*
 * Backward of sum_b <dC_b, C_b> for stl_aa_forward (chain rule; A's side as in stl_backward, B's side as in
 * stl_backward followed by stl_encode_weight_backward, per problem):
 *   dYhat = encode_D(dC)              dD   += Yhat (x) dc
 *   dAhat_b[p] = dYhat_b[p] Bhat_b[p]^T   dA = decode_{E_A}(dAhat)   dE_A += dAhat (x) a
 *   dBhat_b[p] = Ahat_b[p]^T dYhat_b[p]   dB = decode_{E_B}(dBhat)   dE_B += dBhat (x) b
 * dC: (nbatch*m) x n (in).  *_saved: NULL (recomputed) or what stl_aa_forward wrote.  dA, dB: storage dtype
 * (out); dE_A, dE_B, dD: r x 16 fp32 (out), summed over the batch; any output may be NULL.  dBhat is kept in the
 * storage dtype (it is a per-problem intermediate like dAhat, not an accumulated weight gradient).
 * accumulate: as in stl_backward, for dE_A, dE_B, dD.  flags: 0 or STL_FLAG_B_TRANSPOSED, as in the forward call.
 * ws / ws_bytes: at least stl_aa_workspace_bytes(prob, nbatch, STL_OP_BACKWARD).
 */
stl_status_t stl_aa_backward(const stl_problem_t *prob, int64_t nbatch, const void *A, const void *B,
                             const void *E_A, const void *E_B, const void *D, const void *dC,
                             const void *Ahat_saved, const void *Bhat_saved, const void *Yhat_saved, void *dA,
                             void *dB, float *dE_A, float *dE_B, float *dD, int accumulate, void *ws,
                             size_t ws_bytes, int flags, void *stream);

/*
 * Row counts that t does not divide (Class-1 appendix, "More Details on STL Replacement in T2T-ViT", item 1):
 * X is a stack of images with `rows` token rows each (197 in the paper), prob->m = nimg * rows real rows.  Every
 * image is treated as extended with null rows to Mt = ceil(rows/4) tile rows (200 rows); the operator runs on the
 * padded stack, and on the way back the 4 padded output rows of an image's last tile row are combined linearly
 * into its nrho = rows mod 4 remaining real rows with the trainable coefficients `fold` (nrho x 4, fp32, row-major):
 *     C[img*rows + 4(Mt-1) + rho][j] = sum_a fold[rho][a] * Ypad[img*4Mt + 4(Mt-1) + a][j].
 * The paper's case is nrho = 1 (4 coefficients); one combination per remaining row is this library's reading for
 * nrho = 2, 3.  Nothing is copied or padded in memory: null rows are read as zeros inside the encode, the fold is
 * composed into the decoder of the last tile rows, and null rows are never written.  With rows % 4 == 0 the
 * calls equal stl_forward / stl_backward and `fold`, `dfold` are ignored (may be NULL).
 * X: m x k, C: m x n (real rows only).  Plane tensors are over the padded tile rows:
 *   Xhat_save stl_plane_elems(nimg*Mt, K, r), Yhat_save stl_plane_elems(nimg*Mt, N, r) elements, or NULL.
 * rows >= 4 and m % rows == 0 (INVALID_ARG otherwise).
 * ws / ws_bytes: at least stl_ragged_workspace_bytes(prob, rows, STL_OP_FORWARD or STL_OP_BACKWARD).
 * Error behaviour and ownership as for every entry point (see the top of this file); there is no activation flag here.
 */
size_t stl_ragged_workspace_bytes(const stl_problem_t *prob, int64_t rows, int op);
stl_status_t stl_ragged_forward(const stl_problem_t *prob, int64_t rows, const void *X, const void *What,
                                const void *E_X, const void *D, const float *fold, void *C, void *Xhat_save,
                                void *Yhat_save, void *ws, size_t ws_bytes, void *stream);
/*
 * Backward of <dC, C> for stl_ragged_forward: the outputs of stl_backward (gradients of null rows are dropped,
 * null rows count as zeros in dE_X) and dfold (nrho x 4 fp32, or NULL):
 *     dfold[rho][a] = sum_{img,j} dC[img*rows + 4(Mt-1) + rho][j] * Ypad[img*4Mt + 4(Mt-1) + a][j].
 * accumulate applies to dWhat, dE_X, dD and dfold.
 */
stl_status_t stl_ragged_backward(const stl_problem_t *prob, int64_t rows, const void *X, const void *What,
                                 const void *E_X, const void *D, const float *fold, const void *dC,
                                 const void *Xhat_saved, const void *Yhat_saved, void *dX, float *dWhat,
                                 float *dE_X, float *dD, float *dfold, int accumulate, void *ws,
                                 size_t ws_bytes, void *stream);

/* Static text for a status code. */
const char *stl_status_string(stl_status_t status);
/* Text of the last error raised on the calling thread ("" if none).  Thread-local storage. */
const char *stl_last_error(void);
/* Library version, e.g. "0.1.0 gfx950". */
const char *stl_version(void);

#ifdef __cplusplus
}
#endif
#endif /* STL_H_ */
