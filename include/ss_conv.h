/*
 * ss_conv.h -- C ABI of the short causal convolution (+ SiLU) that feeds the selective scan.
 *
 * In the block of arXiv 2312.00752 (Section 3.4, Figure 3) the SSM branch is
 * input projection -> short per-channel convolution -> SiLU -> selective SSM.  The paper
 * names the convolution but gives neither width nor indexing; this library takes it as the
 * left-padded per-channel cross-correlation
 *
 *     v[b,d,t] = bias[d] + sum_{k=0}^{W-1} w[d,k] * x[b,d,t-(W-1)+k]
 *     out      = v * sigmoid(v)  (SS_CONV_SILU)   or   v
 *
 * with x at negative times equal to 0 or, with SS_CONV_HAS_STATE, to the W-1 samples
 * state_in[b,d,:] that preceded the sequence (oldest first).  1 <= W <= SS_CONV_MAX_WIDTH.
 *
 * Rules as in ss_scan.h: device pointers owned by the caller, dense row-major layouts with
 * the sequence axis last, io_dtype tensors 16-byte aligned, float32 ones 4-byte aligned,
 * kernels are only enqueued on `stream`, outputs are overwritten, arguments are validated
 * on the host before any device call, return value SS_OK or a negative SS_ERR_* code of
 * ss_scan.h.  No output may overlap an input.  seqlen == 0 is valid.
 *      x, out, dout, dx     : (B, D, L)    io_dtype
 *      state_in, state_out  : (B, D, W-1)  io_dtype  (ignored when W == 1)
 *      w, dw                : (D, W)       float32
 *      bias, dbias          : (D)          float32
 */
#ifndef SS_CONV_H
#define SS_CONV_H

#include "ss_scan.h"

#ifdef __cplusplus
extern "C" {
#endif

#define SS_CONV_MAX_WIDTH 4

enum {
    SS_CONV_SILU        = 1u, /* apply SiLU to the convolution                              */
    SS_CONV_HAS_BIAS    = 2u, /* bias is given                                              */
    SS_CONV_HAS_STATE   = 4u, /* state_in is given (else the history is zero)               */
    SS_CONV_WRITE_STATE = 8u  /* state_out receives the last W-1 samples seen               */
};

typedef struct {
    int32_t batch, dim, seqlen, width; /* B, D, L, W                                        */
    int32_t io_dtype;                  /* ss_dtype                                          */
    uint32_t flags;                    /* OR of SS_CONV_* bits                              */
    const void *x;                     /* (B,D,L)                                           */
    const float *w, *bias;             /* (D,W), (D)                                        */
    const void *state_in;              /* (B,D,W-1); with SS_CONV_HAS_STATE                 */
    void *out;                         /* (B,D,L)                                           */
    void *state_out;                   /* (B,D,W-1); with SS_CONV_WRITE_STATE               */
} ss_conv_params;

/* Forward: out (and state_out).  Processing a sequence in pieces, each call taking the
 * previous call's state_out as state_in, gives the same result as one call. */
int ss_conv_fwd(const ss_conv_params *p, void *stream);

typedef struct {
    ss_conv_params fwd;   /* the forward call's inputs and flags; out and state_out unread  */
    const void *dout;     /* (B,D,L) io_dtype: gradient w.r.t. out                          */
    void *dx;             /* (B,D,L) io_dtype                                               */
    float *dw;            /* (D,W) float32, summed over batch and time                      */
    float *dbias;         /* (D) float32; required iff SS_CONV_HAS_BIAS                     */
} ss_conv_bwd_params;

/* Backward: recomputes the convolution (nothing is saved by the forward call, as the paper's
 * Appendix D prescribes for the cheap steps of the block) and returns the gradient of
 * <out, dout> w.r.t. x, w and bias; no gradient flows to state_in.  dw and dbias are
 * accumulated with floating-point atomics, so their last bits may differ between runs. */
int ss_conv_bwd(const ss_conv_bwd_params *p, void *stream);

typedef struct {
    int32_t batch, dim, width;
    int32_t io_dtype;
    uint32_t flags;          /* SS_CONV_SILU, SS_CONV_HAS_BIAS                              */
    void *state;             /* (B,D,W-1) io_dtype, updated IN PLACE (oldest sample first)  */
    const void *x_t;         /* (B,D)                                                       */
    const float *w, *bias;
    void *out_t;             /* (B,D)                                                       */
} ss_conv_step_params;

/* One token of the recurrent mode (Section 2): the window slides by one sample. */
int ss_conv_step(const ss_conv_step_params *p, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SS_CONV_H */
