/*
 * ss_layer.h -- C ABI of the selective SSM layer: the steps either side of the scan.
 *
 * Algorithm 2 of arXiv 2312.00752 with the selection functions of Section 3.2 (s_B, s_C
 * linear in the input, Delta through softplus), the low-rank Delta projection of Section 3.6
 * and the convolution / activation / gate of the block in Section 3.4 (Figure 3).  For every
 * batch entry, with the sequence axis last:
 *
 *     u          = SiLU(conv(x))                       (D, L)      ss_conv.h
 *     [r; B; C]  = W_x  @ u                            (R+N+N, L)
 *     delta_raw  = W_dt @ r                            (D, L)
 *     out        = scan(u, softplus(delta_raw + dt_bias), A, B, C, Dskip) * SiLU(z)   ss_scan.h
 *
 * u, [r;B;C] and delta_raw are stored in io_dtype between the steps.  The backward call
 * follows Appendix D ("Memory"): of the forward pass only [r;B;C] (R+2N rows against the 2D
 * rows of x and z) and the scan's checkpoints are kept in `saved`; u and delta_raw are
 * recomputed from x and [r;B;C].
 *
 * Rules as in ss_scan.h (device pointers owned by the caller, dense row-major layouts, io
 * tensors 16-byte aligned, float32 ones 4-byte aligned, outputs overwritten, host-side
 * validation, SS_OK or a negative code).  The two projections and their gradients run on this
 * library's own matrix-core kernels like every other step: no backend library is loaded and no
 * call allocates.  `saved` and `scratch` must be 256-byte aligned; seqlen must be >= 1 and
 * dstate <= SS_MAX_DSTATE.
 *      x, z, out, dout, dx, dz : (B, D, L)     io_dtype
 *      W_x                     : (R+2N, D)     io_dtype   rows: r (R), B (N), C (N)
 *      W_dt                    : (D, R)        io_dtype
 *      conv_w                  : (D, W)        float32;   conv_b, dt_bias, Dskip : (D) float32
 *      A                       : (D, N)        float32
 *      dW_x, dW_dt, dconv_w, dconv_b, ddt_bias, dA, dD : float32, shaped like their parameter
 */
#ifndef SS_LAYER_H
#define SS_LAYER_H

#include "ss_conv.h"
#include "ss_scan.h"

#ifdef __cplusplus
extern "C" {
#endif

#define SS_ERR_BACKEND (-7) /* reserved: no current entry point returns it (there is no backend library) */

typedef struct {
    int32_t batch, dim, seqlen, dstate, dt_rank, conv_width; /* B, D, L, N, R, W             */
    int32_t io_dtype;                                        /* ss_dtype                     */
    uint32_t flags;                                          /* must be 0                    */
    const void *x, *z;
    const float *conv_w, *conv_b;
    const void *W_x, *W_dt;
    const float *dt_bias, *A, *Dskip;
    void *out;
    float *h_last;      /* (B,D,N) float32 or NULL: state after the last token               */
    void *conv_state;   /* (B,D,W-1) io_dtype or NULL: the last W-1 inputs of the conv       */
    void *saved;        /* ss_layer_saved_bytes(): written by the forward call, read by the
                           backward call; NULL in a forward call that no backward follows    */
    size_t saved_bytes;
    void *scratch;      /* ss_layer_scratch_bytes(): free for other use after the call       */
    size_t scratch_bytes;
} ss_layer_params;

/* Sizes of the two buffers; only the shape fields and io_dtype are read.  for_backward
 * selects the scratch size of ss_layer_bwd (larger) or of ss_layer_fwd. */
size_t ss_layer_saved_bytes(const ss_layer_params *p);
size_t ss_layer_scratch_bytes(const ss_layer_params *p, int for_backward);

/* Forward: conv, projections, scan, gate.  h_last and conv_state, if asked for, are what
 * ss_layer_step continues from after a prompt. */
int ss_layer_fwd(const ss_layer_params *p, void *stream);

typedef struct {
    ss_layer_params fwd; /* the forward call's inputs and its `saved`; out is not read;
                            scratch sized for the backward call                              */
    const void *dout;    /* (B,D,L) io_dtype                                                 */
    void *dx, *dz;       /* (B,D,L) io_dtype                                                 */
    float *dconv_w, *dconv_b, *dW_x, *dW_dt, *ddt_bias, *dA, *dD;
} ss_layer_bwd_params;

/* Backward: gradient of <out, dout> w.r.t. x, z and every parameter. */
int ss_layer_bwd(const ss_layer_bwd_params *p, void *stream);

typedef struct {
    int32_t batch, dim, dstate, dt_rank, conv_width; /* B, D, N, R, W                        */
    int32_t io_dtype;
    uint32_t flags;                                  /* must be 0                            */
    float *h;                  /* (B,D,N) float32 state, updated IN PLACE                    */
    void *conv_state;          /* (B,D,W-1) io_dtype window, updated IN PLACE                */
    const void *x_t, *z_t;     /* (B,D)                                                      */
    const float *conv_w, *conv_b;
    const void *W_x, *W_dt;
    const float *dt_bias, *A, *Dskip;
    void *out_t;               /* (B,D)                                                      */
    void *scratch;             /* ss_layer_step_scratch_bytes(), 256-byte aligned            */
    size_t scratch_bytes;
} ss_layer_step_params;

size_t ss_layer_step_scratch_bytes(const ss_layer_step_params *p);

/* One token of the layer in recurrent mode (Section 2): the conv window slides by one sample,
 * the projections become (B, D) x (D, R+2N) and (B, R) x (R, D) products, and Eq. 2a/2b are
 * applied once; constant time and memory per token.  bf16 calls with D % 32 == 0, R % 8 == 0,
 * R <= 256, N <= 16 and 16-byte aligned W_x, W_dt and h take three launches (both projections
 * on the matrix cores, delta_t formed inside the state update); other calls form the two
 * products with the general projection kernel first.  Deterministic either way. */
int ss_layer_step(const ss_layer_step_params *p, void *stream);

/* The products behind the layer's projections (Algorithm 2: the linear maps s_B, s_C of
 * Section 3.2 and the low-rank Delta projection of Section 3.6) and their gradients, callable
 * on their own:
 *     C[i] (M x N) = op(A[i]) (M x K)  op(B[i]) (K x N)   [+ C[i] with SS_GEMM_ACCUMULATE],  i < batch,
 * accumulated in float32.  Element (m, k) of op(A[i]) is A[i * a_batch + m * a_m + k * a_k] and
 * element (k, n) of op(B[i]) is B[i * b_batch + k * b_k + n * b_n] (strides in elements, so either
 * operand may be stored transposed; a batch stride of 0 shares an operand); C is row-major with
 * row pitch ldc, float32 with SS_GEMM_C_FLOAT and in io_dtype otherwise.  A and B are io_dtype.
 * bf16 products of the layer's three shapes (few output rows with a long contraction over the rows
 * of B; many output rows with a contraction of at most 160; both operands contiguous along the
 * contraction index with a float32 result) run on matrix-core kernels when sizes are multiples of
 * 64 (rows / columns of the big side), 16 (the small side, at most 160) and pointers and strides
 * are multiples of 16 bytes; everything else, and every call with SS_GEMM_GENERAL, runs on a
 * general kernel.  `workspace` is optional device memory (256-byte aligned) that the call may
 * overwrite: with ss_proj_gemm_workspace_bytes(p) bytes of it, a product of the first shape with
 * fewer than 512 column tiles x batch entries and K >= 4096, a multiple of 512, splits its
 * contraction over two workgroups per tile (float32 shares, summed by a second kernel); the
 * result may then differ from the unsplit one in the last bf16 digit.  Device pointers; C must not overlap A or B.  SS_OK, SS_ERR_NULL,
 * SS_ERR_SHAPE (negative size), SS_ERR_UNSUPPORTED (dtype, unknown flag, more than 65535 batch
 * entries or 64-row tiles) or SS_ERR_LAUNCH. */
#define SS_GEMM_C_FLOAT    1u
#define SS_GEMM_ACCUMULATE 2u
#define SS_GEMM_GENERAL    4u
typedef struct {
    int32_t M, N, K, batch;
    int32_t io_dtype;           /* ss_dtype of A and B (and of C without SS_GEMM_C_FLOAT)         */
    uint32_t flags;             /* SS_GEMM_*                                                      */
    const void *A;
    int64_t a_m, a_k, a_batch;
    const void *B;
    int64_t b_k, b_n, b_batch;
    void *C;
    int64_t ldc, c_batch;
    void *workspace;            /* optional, see above; NULL: never split                        */
    size_t workspace_bytes;
} ss_gemm_params;
int ss_proj_gemm(const ss_gemm_params *p, void *stream);
/* Bytes of workspace with which ss_proj_gemm may split the contraction of *p (reads M, N, batch;
 * 0 for a NULL or negative-size argument).  Smaller or absent workspaces are valid: no split. */
size_t ss_proj_gemm_workspace_bytes(const ss_gemm_params *p);

#ifdef __cplusplus
}
#endif
#endif /* SS_LAYER_H */
