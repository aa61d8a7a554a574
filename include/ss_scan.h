/*
 * ss_scan.h -- C ABI of the MI355X (gfx950) selective-scan library.
 *
 * The operation is the selective state-space recurrence of arXiv 2312.00752
 * (Algorithm 2, steps 5-6; Eq. 2a/2b; Eq. 4), fused as the paper's Section 3.3.2 /
 * Appendix D describe: the expanded (B,L,D,N) quantities live on chip only.
 * For every batch b and channel d independently (diagonal A, Section 2):
 *
 *     r_t      = delta[b,d,t] (+ delta_bias[d])
 *     dt_t     = softplus(r_t)            if SS_DELTA_SOFTPLUS, else r_t   (Section 3.2, tau_Delta)
 *     abar_t,n = exp(dt_t * A[d,n])                                        (Eq. 4)
 *     h_t,n    = abar_t,n * h_{t-1,n} + phi_t,n * Bmat[b,n,t] * u[b,d,t]   (Eq. 2a)
 *                phi_t,n = dt_t                          (default: first-order B-bar)
 *                phi_t,n = (abar_t,n - 1) / A[d,n]       (SS_EXACT_ZOH_B: the B-bar of Eq. 4;
 *                                                         dt_t where A[d,n] == 0)
 *     y_t      = sum_n Cmat[b,n,t] * h_t,n (+ Dskip[d] * u[b,d,t])         (Eq. 2b)
 *     out_t    = y_t * z_t * sigmoid(z_t) if SS_HAS_Z, else y_t            (Section 3.4 gate)
 *
 * with h_{-1} = h0[b,d,:] (SS_HAS_H0) or 0, and h_last = h_{L-1}.
 *
 * With SS_COMPLEX_STATE the state h, A, Bmat and Cmat are complex and the same equations are
 * taken over the complex numbers, with first-order B-bar and the real part read out:
 *     abar = exp(dt A),  h_t = abar h_{t-1} + dt Bmat u,  y_t = Re(sum_n Cmat h_t,n) (+ Dskip u).
 * dstate counts complex states.  Every complex array carries a (re, im) pair where the real
 * case has one number, as the axis right after n: A, dA (D,N,2); h0, h_last, dh_last, dh0
 * (B,D,N,2); Bmat, Cmat, dB, dC (B,N,2,L) (a row of real parts, then a row of imaginary
 * parts, per state); a time-invariant Bmat / Cmat (D,N,2).  Gradients of complex inputs are
 * (dLoss/dRe, dLoss/dIm).  SS_EXACT_ZOH_B is not available together with it.
 *
 * General rules for every entry point
 *  - All data pointers are DEVICE pointers owned by the caller.  The library never
 *    allocates, frees or synchronises; a call only enqueues kernels on `stream`
 *    (a hipStream_t passed as void*; NULL is the default stream).  The parameter
 *    struct itself is host memory and is read before the call returns.
 *  - Layouts are dense row-major with the sequence axis last:
 *      u, delta, z, out, dout, du, ddelta, dz : (B, D, L)  in io_dtype
 *      Bmat, Cmat                             : (B, N, L)  in io_dtype
 *      dB, dC                                 : (B, N, L)  float32
 *        (with SS_B_FIXED / SS_C_FIXED: Bmat, dB / Cmat, dC are (D, N) float32, like A)
 *      A, dA                                  : (D, N)     float32
 *      Dskip, delta_bias, dD, ddelta_bias     : (D)        float32
 *      h0, h_last, dh_last, dh0               : (B, D, N)  float32
 *    State, abar and every accumulation are float32 whatever io_dtype is.
 *  - Every io_dtype base pointer must be 16-byte aligned, float32 ones 4-byte aligned.
 *  - Outputs are overwritten, never accumulated into.  Inputs are not modified.
 *  - Return value: SS_OK (0) or a negative SS_ERR_* code.  Arguments are validated on
 *    the host before any device call, so a rejected call has touched nothing.
 *    seqlen == 0 is valid: tensors with a zero-length axis may then be NULL, h_last (if
 *    requested) receives h0 or 0, and the backward call returns zero parameter gradients
 *    and dh0 = dh_last.
 *  - Supported: 1 <= dstate <= SS_MAX_DSTATE, io_dtype in {SS_F32, SS_BF16}.  The kernels hold
 *    16 states per row on chip; more states are handled 16 at a time in passes over the
 *    sequence that add up in the output (time and checkpoint size grow with ceil(dstate/16),
 *    io_dtype sums are rounded once per pass, and a gated forward call then needs the
 *    workspace even without SS_SAVE_FOR_BWD).
 */
#ifndef SS_SCAN_H
#define SS_SCAN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SS_MAX_DSTATE 256
/* Spacing, in time steps, of the state checkpoints the forward pass leaves for the
 * backward pass (Appendix D: states are recomputed, not stored). */
#define SS_CHECKPOINT_STEPS 16

typedef enum { SS_F32 = 0, SS_BF16 = 1 } ss_dtype;

enum {
    SS_DELTA_SOFTPLUS = 1u,  /* dt = softplus(delta + bias) instead of delta + bias        */
    SS_HAS_DELTA_BIAS = 2u,  /* delta_bias is given                                        */
    SS_HAS_D          = 4u,  /* Dskip is given                                             */
    SS_HAS_Z          = 8u,  /* z is given: multiplicative SiLU gate                       */
    SS_HAS_H0         = 16u, /* h0 is given (else the scan starts from the zero state)     */
    SS_WRITE_H_LAST   = 32u, /* h_last is written                                          */
    SS_SAVE_FOR_BWD   = 64u, /* forward: leave state checkpoints in `workspace`            */
    SS_EXACT_ZOH_B    = 128u, /* exact zero-order-hold B-bar of Eq. 4 instead of dt * B    */
    SS_B_FIXED        = 256u, /* Bmat is the time-invariant (D,N) float32 parameter of
                                 Algorithm 1 (the non-selective arm of Table 7); dB likewise */
    SS_C_FIXED        = 512u, /* the same for Cmat / dC                                     */
    SS_COMPLEX_STATE  = 1024u /* complex state (Section 3.6, "Real vs. Complex"): see below */
};

enum {
    SS_OK = 0,
    SS_ERR_NULL = -1,        /* a required pointer (or one implied by a flag) is NULL      */
    SS_ERR_SHAPE = -2,       /* batch, dim or dstate < 1, or seqlen < 0                    */
    SS_ERR_UNSUPPORTED = -3, /* dstate > SS_MAX_DSTATE, unknown io_dtype or unknown flag   */
    SS_ERR_ALIGN = -4,       /* a base pointer is not aligned as stated above              */
    SS_ERR_WORKSPACE = -5,   /* workspace missing or smaller than ss_workspace_bytes()     */
    SS_ERR_LAUNCH = -6       /* the HIP runtime refused a launch                           */
};

typedef struct {
    int32_t batch, dim, seqlen, dstate; /* B, D, L, N                                      */
    int32_t io_dtype;                   /* ss_dtype of u, delta, z, Bmat, Cmat, out (and of
                                           dout, du, ddelta, dz in the backward call)      */
    uint32_t flags;                     /* OR of SS_* flag bits                            */
    const void *u, *delta, *z;          /* (B,D,L); z only with SS_HAS_Z                   */
    const void *Bmat, *Cmat;            /* (B,N,L)                                         */
    const float *A;                     /* (D,N)                                           */
    const float *Dskip, *delta_bias;    /* (D); with SS_HAS_D / SS_HAS_DELTA_BIAS          */
    const float *h0;                    /* (B,D,N); with SS_HAS_H0                         */
    void *out;                          /* (B,D,L)                                         */
    float *h_last;                      /* (B,D,N); with SS_WRITE_H_LAST                   */
    void *workspace;                    /* scratch the caller lends; see below             */
    size_t workspace_bytes;
} ss_fwd_params;

/* Bytes of workspace a call with these sizes needs: for_backward == 0 for a plain
 * ss_scan_fwd, 1 for ss_scan_fwd with SS_SAVE_FOR_BWD and the ss_scan_bwd that follows
 * it.  Read: batch, dim, seqlen, dstate, io_dtype and the flags SS_HAS_Z, SS_B_FIXED,
 * SS_C_FIXED and SS_COMPLEX_STATE (they change the number of state slots, add partial-sum
 * blocks for a time-invariant operand's gradient, and decide whether B and C are repacked and
 * the sequence split), so pass the flags of the call the workspace is for.  The
 * content is opaque (state checkpoints every SS_CHECKPOINT_STEPS steps, the pre-gate
 * output when there is a gate, per-segment carries when a long sequence with few rows is
 * split across workgroups, and partial sums of the backward pass); a forward call with
 * SS_SAVE_FOR_BWD fills it and the matching backward call must get the same, untouched
 * buffer.  256-byte alignment is required.  Returns 0 when none is needed.
 * A plain forward call (for_backward == 0) never requires a workspace: the size returned
 * for it is scratch that, if lent, lets the library read B and C from a repacked copy
 * (selective B and C, real state) and split a long sequence with few rows across
 * workgroups; without it the call is correct but slower and runs one workgroup per 64
 * rows.  (More than 16 states with a gate are the exception: the pre-gate output is
 * accumulated in the workspace, which is then required.) */
size_t ss_workspace_bytes(const ss_fwd_params *p, int for_backward);

/* Forward scan (Algorithm 2 steps 5-6 with the fusion of Appendix D).  Writes out, and
 * h_last / checkpoints according to the flags. */
int ss_scan_fwd(const ss_fwd_params *p, void *stream);

/* The plain forward scan for callers that cannot allocate device memory and have no workspace
 * to lend: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same operation, arguments and results as ss_scan_fwd without SS_SAVE_FOR_BWD, but the scratch
 * that ss_workspace_bytes(p, 0) describes (repacked B and C, per-segment states of a split
 * sequence, the pre-gate accumulator of more than 16 states) is a fixed array of
 * SS_STATIC_SCRATCH_BYTES in the library's own device image instead of p->workspace, which is
 * ignored.  The call allocates nothing and frees nothing; the array's device address is looked up
 * once per device, on the first call there.
 *  - SS_SAVE_FOR_BWD is rejected with SS_ERR_UNSUPPORTED (the backward pass needs a workspace
 *    that outlives the call), a problem whose scratch exceeds SS_STATIC_SCRATCH_BYTES with
 *    SS_ERR_WORKSPACE; both before anything is enqueued.
 *  - Every call on a GPU uses that GPU's one array: calls that overlap on one GPU (different
 *    streams, or graphs replayed concurrently) race.  Calls in stream order are safe; nothing
 *    in the array has to survive from one call to the next. */
#define SS_STATIC_SCRATCH_BYTES (64u << 20)
int ss_scan_fwd_static(const ss_fwd_params *p, void *stream);

typedef struct {
    ss_fwd_params fwd;        /* the forward call's inputs, flags and filled workspace;
                                 fwd.out and fwd.h_last are not read                       */
    const void *dout;         /* (B,D,L) io_dtype: gradient of the loss w.r.t. out         */
    const float *dh_last;     /* (B,D,N) or NULL: gradient w.r.t. h_last                   */
    void *du, *ddelta, *dz;   /* (B,D,L) io_dtype; dz required iff SS_HAS_Z                */
    float *dB, *dC;           /* (B,N,L) float32, summed over channels                     */
    float *dA;                /* (D,N) float32, summed over batch and time                 */
    float *dD, *ddelta_bias;  /* (D) float32; required iff SS_HAS_D / SS_HAS_DELTA_BIAS    */
    float *dh0;               /* (B,D,N) float32 or NULL: gradient w.r.t. h0               */
} ss_bwd_params;

/* Backward scan: recomputes the states chunk by chunk from the forward pass's
 * checkpoints (Appendix D, "Memory") and returns the gradient of
 * <out, dout> + <h_last, dh_last> w.r.t. every input.  dB and dC are accumulated with
 * floating-point atomics, so their last bits may differ between runs. */
int ss_scan_bwd(const ss_bwd_params *p, void *stream);

typedef struct {
    int32_t batch, dim, dstate;       /* B, D, N                                           */
    int32_t io_dtype;                 /* of u_t, delta_t, z_t, B_t, C_t, out_t             */
    uint32_t flags;                   /* SS_DELTA_SOFTPLUS, SS_HAS_DELTA_BIAS, SS_HAS_D,
                                         SS_HAS_Z, SS_EXACT_ZOH_B, SS_B_FIXED, SS_C_FIXED,
                                         SS_COMPLEX_STATE                                   */
    float *h;                         /* (B,D,N) float32 state, updated IN PLACE           */
    const void *u_t, *delta_t, *z_t;  /* (B,D)                                             */
    const void *B_t, *C_t;            /* (B,N); (D,N) float32 with SS_B_FIXED / SS_C_FIXED */
    const float *A, *Dskip, *delta_bias;
    void *out_t;                      /* (B,D)                                             */
} ss_step_params;

/* One token of the recurrent mode (Section 2, Eq. 2a/2b applied once): constant work
 * per step, no cache of earlier tokens.  h must be 16-byte aligned. */
int ss_step(const ss_step_params *p, void *stream);

/* Static, NUL-terminated description of a return code. */
const char *ss_strerror(int code);

/* Library version: major * 10000 + minor * 100 + patch. */
int ss_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SS_SCAN_H */
