// Internal launcher interface between the C ABI (stl_api.hip) and the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace stl {

// dtype: 0 = fp32 storage, 1 = bf16 storage (matches stl_dtype_t)
// pg: rows per group of the plane tensor's layout (see plane_row_base); 0 = plane-major (one group of all rows)
constexpr int kPlaneGroup = 64;   // group size of the activation-side plane tensors

// Which matrix rows lie behind a tile row of the plane tensors.
//   plain  (Mt == 0): tile row I covers matrix rows 4I .. 4I+3.
//   ragged (Mt > 0):  the matrix is a stack of images with `rows` real rows each (197 tokens in the Class-1 appendix),
//     thought of as padded with null rows to Mt = ceil(rows / 4) tile rows per image.  Tile row I = img * Mt + l covers
//     matrix rows img * rows + 4l + a for the a with 4l + a < rows; the other entry rows are null rows: they read as
//     zero and are never written.  Only the last tile row of an image can be incomplete.
// A launch walks over a selection of the tile rows: all of them, only the complete-by-position ones (every tile row
// but the last of each image), or only the last of each image.
struct RowMap {
    int Mt = 0, rows = 0;
    int sel = 0;                       // 0: all tile rows, 1: all but each image's last, 2: each image's last
    __host__ __device__ __forceinline__ int tile_row(int idx) const
    {
        if (Mt == 0 || sel == 0) return idx;
        if (sel == 1) return idx + idx / (Mt - 1);
        return idx * Mt + Mt - 1;
    }
    __host__ __device__ __forceinline__ size_t row0(int I) const
    {
        if (Mt == 0) return (size_t)I * 4;
        const int img = I / Mt;
        return (size_t)img * rows + (size_t)(I - img * Mt) * 4;
    }
    __host__ __device__ __forceinline__ int valid(int I) const       // real entry rows of tile row I (1..4)
    {
        if (Mt == 0) return 4;
        const int left = rows - (I % Mt) * 4;
        return left < 4 ? left : 4;
    }
    // number of tile rows a launch with this selection walks over, R = all tile rows
    __host__ __device__ __forceinline__ int count(int R) const
    {
        if (Mt == 0 || sel == 0) return R;
        return sel == 1 ? R / Mt * (Mt - 1) : R / Mt;
    }
};

// planes P[p][R][Cc] <- encoder E (r x 16) applied to every 4x4 tile of A (4R x 4Cc)
// rm: which matrix rows lie behind the tile rows, and which tile rows the launch walks over (R always counts ALL tile
// rows of the plane tensor); basis_f32: E (or Dm) is stored as fp32 whatever the dtype
hipError_t launch_encode(int dtype, const void *A, const void *E, void *P, int R, int Cc, int r, int pg, hipStream_t s,
                         RowMap rm = RowMap(), bool basis_f32 = false);
// matrix Cmat (4R x 4Cc) <- decoder Dm^T (r x 16 stored) applied to planes P[p][R][Cc]
hipError_t launch_decode(int dtype, const void *P, const void *Dm, void *Cmat, int R, int Cc, int r, bool gelu, int pg,
                         hipStream_t s, RowMap rm = RowMap(), bool basis_f32 = false);

// G[p][q] (+)= sum_tiles P[p][tile] * tileview(V)[tile][q]; `part` holds outer_reduce_blocks(R*Cc) * r * 16 floats
int outer_reduce_blocks(int64_t tiles);
hipError_t launch_outer_reduce(int dtype, const void *P, const void *V, float *G, float *part, int R, int Cc, int r,
                               int accumulate, int pg, hipStream_t s, RowMap rm = RowMap());

// decode and basis gradient in one pass over the planes (bf16): Cmat <- decode(P, Dm), G (+)= P . tileview(V);
// `part` holds decode_outer_blocks(R, Cc) * r * 16 floats
bool decode_outer_eligible(int dtype, int Cc);
int decode_outer_blocks(int R, int Cc);
hipError_t launch_decode_outer(const void *P, const void *Dm, void *Cmat, const void *V, float *G, float *part, int R,
                               int Cc, int r, int accumulate, int pg, hipStream_t s, RowMap rm = RowMap(), bool final_sum = true);

// G[i] (+)= sum over nb partials part[b][i], i < n_out, in block order (second stage of the basis-gradient sums)
hipError_t launch_outer_final(const float *part, float *G, int nb, int n_out, int accumulate, hipStream_t s);
// two such sums in one launch (final_sum = false in the two fused passes leaves their partials for this)
hipError_t launch_outer_final_pair(const float *part0, float *G0, int nb0, const float *part1, float *G1, int nb1, int n_out,
                                   int accumulate, hipStream_t s);

// encode and basis gradient in one pass over the matrix (bf16): P <- encode(A, E), G (+)= Qp . tileview(A);
// `part` holds encode_outer_blocks(R, Cc) * r * 16 floats
bool encode_outer_eligible(int dtype, int Cc);
int encode_outer_blocks(int R, int Cc);
hipError_t launch_encode_outer(const void *A, const void *E, void *P, const void *Qp, float *G, float *part, int R, int Cc,
                               int r, int accumulate, int pg, hipStream_t s, RowMap rm = RowMap(), bool final_sum = true);

// fold of an image's last tile row (row counts not divisible by 4): composed decoder Dp (r x 16 fp32) from Dm and the
// nrho x 4 fold coefficients; and the gradients that come from those tile rows, given Gt = Yhat (x) dC over them
hipError_t launch_fold_decoder(int dtype, const void *Dm, const float *fold, float *Dp, int r, int nrho, hipStream_t s);
hipError_t launch_fold_grads(int dtype, const float *Gt, const void *Dm, const float *fold, float *dD, float *dfold, int r,
                             int nrho, int accumulate, hipStream_t s);

// Et[p][4a+b] = E[p][4b+a] (storage type): the basis that encodes B^T when applied to the tiles of B; and the same map
// on a gradient, G[p][4a+b] (+)= Gt[p][4b+a] (fp32)
hipError_t launch_transpose_basis(int dtype, const void *E, void *Et, int r, hipStream_t s);
hipError_t launch_transpose_basis_grad(const float *Gt, float *G, int r, int accumulate, hipStream_t s);

// bf16 encode with whole-line plane stores (Cc % 8 == 0); launch_encode picks it
hipError_t launch_encode_lines(const void *A, const void *E, void *P, int R, int Cc, int r, int pg, hipStream_t s, RowMap rm);

// out[i] = bf16(in[i]), round to nearest even
hipError_t launch_cast_bf16(const float *in, void *out, size_t n, hipStream_t s);

// inter-layer step of two stacked layers in one pass (bf16): Q[s] <- encode_{E2}( act( decode_{Dm}(P) ) ), planes P
// r1 x R x Cc -> planes Q r2 x R x Cc, the hidden activation never stored
bool recode_eligible(int dtype, int Cc);
hipError_t launch_recode(const void *P, const void *Dm, const void *E2, void *Q, int R, int Cc, int r1, int r2, bool gelu,
                         int pg, hipStream_t s);

// Batched plane products  Out[b][p][i][j] (+)= sum_l A[b][p](i,l) * B[b][p](l,j),  p < batch, b < nb, dense planes.
struct GemmDesc {
    int Mi, Nj, Kl;   // output rows, output columns, contraction length (all in tiles of the STL problem)
    int batch;        // number of planes r
    bool a_kmajor;    // false: A[p] stored [i][l] (l contiguous);  true: stored [l][i] (i contiguous)
    bool b_kmajor;    // true:  B[p] stored [l][j] (j contiguous);  false: stored [j][l] (l contiguous)
    bool out_f32;     // output stored as fp32 regardless of dtype (weight gradient)
    bool accumulate;  // Out += result (only with out_f32)
    // layout of each operand: rows per group (see plane_row_base), counted in the operand's stored rows -- i for A
    // stored [i][l], l for A stored [l][i], and so on; 0 = plane-major
    int a_pg = 0, b_pg = 0, o_pg = 0;
    // nb independent problems of this shape stacked along the stored rows of every operand: problem b owns stored rows
    // [b * rows, (b + 1) * rows) of A, B and Out (rows = the operand's stored row count for one problem)
    int nb = 1;
    int a_rows() const { return a_kmajor ? Kl : Mi; }
    int b_rows() const { return b_kmajor ? Kl : Nj; }
    int a_rows_per_group() const { return a_pg > 0 ? a_pg : nb * a_rows(); }
    int b_rows_per_group() const { return b_pg > 0 ? b_pg : nb * b_rows(); }
    int o_rows_per_group() const { return o_pg > 0 ? o_pg : nb * Mi; }
};
hipError_t launch_plane_gemm(int dtype, const GemmDesc &g, const void *A, const void *B, void *Out, hipStream_t s);
// the any-shape path (fp32 MFMA), also used directly for fp32 storage
hipError_t launch_plane_gemm_generic(int dtype, const GemmDesc &g, const void *A, const void *B, void *Out,
                                     hipStream_t s);
// bf16 MFMA path; returns false in *ok if the shape is not eligible (caller falls back)
bool plane_gemm_mfma_eligible(const GemmDesc &g);
hipError_t launch_plane_gemm_mfma(const GemmDesc &g, const void *A, const void *B, void *Out, hipStream_t s);
// bf16 MFMA path with LDS-DMA loads and a multi-stage LDS ring (large planes, contraction % 32 == 0)
bool plane_gemm_pipe_eligible(const GemmDesc &g);
hipError_t launch_plane_gemm_pipe(const GemmDesc &g, const void *A, const void *B, void *Out, hipStream_t s);

// The whole forward pass as one persistent launch: encode and decode items run on some CUs while the plane products
// run on the others (bf16, r <= 32; see stl_pipeline.hip).  `counters` is forward_pipeline_counter_bytes(M) bytes of
// scratch (cleared by the launch itself).  Results are bit-identical to encode -> plane products -> decode.
bool forward_pipeline_eligible(int dtype, int M, int K, int N, int r);
size_t forward_pipeline_counter_bytes(int M);
hipError_t launch_forward_pipeline(const void *X, const void *E, const void *What, const void *Dm, void *Xhat, void *Yhat,
                                   void *C, void *counters, int M, int K, int N, int r, bool gelu, hipStream_t s);

// the same with the first ([row][l]) operand fetched as whole 128-byte lines (contraction a multiple of 64, one problem)
bool plane_gemm_wide_eligible(const GemmDesc &g);
hipError_t launch_plane_gemm_wide(const GemmDesc &g, const void *A, const void *B, void *Out, hipStream_t s);

// Forward on one output block with all planes resident (decode in the epilogue).  encode_in_kernel: Xin is X
// (single-launch fused form); otherwise Xin is Xhat.  Ysave may be NULL.  bf16 storage only.
bool block_forward_eligible(int dtype, int M, int K, int N, int r);
hipError_t launch_block_forward(bool encode_in_kernel, const void *Xin, const void *What, const void *E, const void *Dm,
                                void *C, void *Ysave, int M, int K, int N, int r, bool gelu, int pg, hipStream_t s);

}  // namespace stl
