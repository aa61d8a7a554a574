// Internal interface between the C-ABI entry points (ss_api.hip) and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ss_scan.h"

namespace ss {

enum : uint32_t {
    F_DELTA_SOFTPLUS = SS_DELTA_SOFTPLUS,
    F_HAS_DELTA_BIAS = SS_HAS_DELTA_BIAS,
    F_HAS_D = SS_HAS_D,
    F_HAS_Z = SS_HAS_Z,
    F_HAS_H0 = SS_HAS_H0,
    F_EXACT_ZOH_B = SS_EXACT_ZOH_B,
    F_COMPLEX = SS_COMPLEX_STATE,
    F_B_FIXED = SS_B_FIXED,
    F_C_FIXED = SS_C_FIXED,
};

struct FwdArgs {
    int B, D, L, N;
    // More than 16 states are handled 16 at a time: N is the size of the group this launch
    // covers, NS the total number of states = the stride of every (..., n) array, whose
    // pointers (A, h0, h_last, Bm, Cm and the gradients) already point at the group's first state.
    int NS;
    int acc_y;  // forward: this group's C*h is added to the y an earlier group left in ysave (or in out)
    // Fewer than 16 states on the common path (real state, first-order B-bar, selective B / C, L % 8 == 0):
    // the states are dealt out to the waves in turn -- slot k of wave w is state 4k + w instead of
    // 4w + k -- so that every wave (every SIMD) carries its share and the kernels can be built for
    // ceil(N / 4) slots per lane; the cost then follows the state size (Table 10).  The 16-float records of
    // the workspace (checkpoints, segment states and carries, dA partials) stay in slot order 4w + k.
    int il;
    uint32_t flags;
    int vec_ok;  // L % 8 == 0: every row starts 16-byte aligned and 8-step slices are whole or empty
    const void *u, *delta, *z, *Bm, *Cm;
    long bc_bstride;  // elements between consecutive batch entries of Bm and Cm (N * L when dense)
    // Staged copy of the selective B and C for the forward kernels, or null.  In the io dtype,
    // packed per wave: [B][4 * ceil(NS / 16)][Lp / 4][B: 4 states x 4 steps | C: 4 states x 4 steps],
    // Lp = L rounded up to a whole chunk, zeros for states past NS and steps past L.  What one
    // wave needs for a group of 4 steps is then one contiguous 64- (bf16) or 128-byte piece.
    const void* bcs;
    int Lp;
    // Layer forward, bf16: instead of reading delta, the kernel forms delta_raw = W_dt r on the
    // matrix cores.  W_dt (D, R) row-major; rT (B, Lp, Rp): r transposed, zero-padded to Rp = R
    // rounded up to 32 and to Lp steps.  Null W_dt: delta is read from memory.
    const void *W_dt, *rT;
    int R, Rp;
    const float *A, *Dskip, *bias, *h0;
    void* out;
    float* h_last;  // may be null
    float* ckpt;    // [checkpoint][B][D][16]: state entering every 16-step block, or null
    void* ysave;    // (B,D,L) io dtype: y before the gate, kept for the backward pass, or null
    // Split of the sequence across workgroups (few rows, long L).  Segment s covers steps
    // [s*seg_len, min(L, (s+1)*seg_len)); seg_len is a multiple of 32.  nseg == 1: no split.
    int seg_len, nseg;
    float* seg_h;      // [nseg][B][D][16]: local end state of a segment, then its incoming state
    float* seg_sumdt;  // [nseg][B][D]: sum of the step sizes of a segment
};

struct BwdArgs {
    FwdArgs f;  // out / h_last unused; ckpt required
    int acc;           // du, ddelta and dbias of an earlier state group are already there: add to them
    long dbc_bstride;  // elements between consecutive batch entries of dB and dC (NS * L)
    const void* dout;
    const float* dh_last;
    void *du, *ddelta, *dz;
    float *dB, *dC;             // (B,N,L), zeroed before the scan kernel, atomically accumulated;
                                // (D,N), written by the reduction kernel, for a time-invariant B / C
    float *dBf_part, *dCf_part; // [B][D][16] per-batch partial sums of a time-invariant B's / C's gradient
    float *dA_part;             // [nseg][B][D][16] partial sums per segment and batch entry
    float *dD_part, *db_part;   // [nseg][B][D]
    float* seg_g;               // [nseg][B][D][16]: adjoint carry of a segment (local, then incoming)
    float* dh0;
    float *dA, *dD, *dbias;     // final outputs of the reduction kernel
};

constexpr int STEP_NPARTS = 4;   // partial results the layer's decode projection leaves for the step kernel

struct StepArgs {
    int B, D, N;   // N: all states (the step kernels loop over them; no groups)
    uint32_t flags;
    float* h;
    const void *u_t, *delta_t, *z_t, *B_t, *C_t;
    long bc_stride;  // elements between consecutive batch rows of B_t and C_t (N when dense)
    // Layer decode: instead of delta_t, B_t, C_t the kernel takes the float32 projection output
    // P (B, ldp) = [r (R); B (N); C (N)], given as the sum of STEP_NPARTS partial results B * ldp
    // floats apart, and W_dt (D, R) in the io dtype; it adds the parts, rounds to the io dtype (the
    // layer stores its projection so) and forms delta_t = W_dt r itself.  Null: not used.
    const float* P;
    const void* W_dt;
    int R, ldp;
    const float *A, *Dskip, *bias;
    void* out_t;
};

// Each returns 0, or -1 if the runtime refused a launch.  io_dtype: 0 = float, 1 = bf16.
int launch_fwd(const FwdArgs& a, int io_dtype, hipStream_t stream);
// fills the staged copy `bcs` (all NS states) from a.Bm and a.Cm
int launch_stage_bc(const FwdArgs& a, void* bcs, int io_dtype, hipStream_t stream);
int launch_bwd(const BwdArgs& a, int io_dtype, hipStream_t stream);
int launch_step(const StepArgs& a, int io_dtype, hipStream_t stream);
int launch_step_projected(const StepArgs& a, hipStream_t stream);   // bf16 I/O only

// The public scan entry points with one extra degree of freedom: B and C of batch entry b
// start b * bc_bstride elements after Bmat / Cmat (the public calls pass dstate * seqlen).
// Validation and return codes are those of ss_scan_fwd / ss_scan_bwd.
int scan_fwd_strided(const ss_fwd_params* p, long bc_bstride, void* stream);
// The same with delta_raw = W_dt r formed inside the scan kernel (bf16): W_dt (D, R) row-major,
// rT (B, Lp, Rp) = r transposed and zero-padded, Lp = L rounded up to 32, Rp = R rounded up to 32;
// p->delta is not read.  Returns SS_ERR_UNSUPPORTED, before anything is enqueued, when the call
// does not qualify (then use scan_fwd_strided with delta in memory).
int scan_fwd_fused(const ss_fwd_params* p, long bc_bstride, const void* W_dt, int R, const void* rT, void* stream);
bool scan_fwd_fusable(const ss_fwd_params* p, int R);   // whether scan_fwd_fused would take the call
int scan_bwd_strided(const ss_bwd_params* p, long bc_bstride, void* stream);
// ss_step with B_t / C_t rows bc_stride elements apart (the public call passes dstate).
int step_strided(const ss_step_params* p, long bc_stride, void* stream);

// ss_step for the layer's decode: delta_t, B_t, C_t come from the float32 projection output
// P (B, ldp) = [r; B; C] and W_dt (D, R) (see StepArgs); p's delta_t, B_t, C_t are ignored.
int step_projected(const ss_step_params* p, const float* P, const void* W_dt, int R, int ldp, void* stream);

// C[i] (M x N, row pitch ldc) = op(A[i]) (M x K) op(B[i]) (K x N) [+ C[i]] for i < batch, float
// accumulation.  Element (m, k) of op(A[i]) is A[i * a_batch + m * a_m + k * a_k], element (k, n) of
// op(B[i]) is B[i * b_batch + k * b_k + n * b_n] (strides in elements, so either operand may be stored
// transposed).  A and B are bf16 or float (bf16); C is float if c_float, else like A and B.
struct GemmArgs {
    int M, N, K, batch;
    const void* A; long a_m, a_k, a_batch;
    const void* B; long b_k, b_n, b_batch;
    void* C; long ldc, c_batch;
    bool bf16, c_float, accumulate;
    bool general;   // take the general kernel even where a matrix-core kernel fits (for verification)
    // optional device memory for float32 shares of the result (up to 4 * batch * M * N floats are used): lets a
    // product with few output rows and few columns split its contraction across workgroups
    void* split_ws;
    size_t split_ws_bytes;
};
int gemm(const GemmArgs& g, hipStream_t stream);
}  // namespace ss
