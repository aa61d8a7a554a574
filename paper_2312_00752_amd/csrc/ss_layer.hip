// Selective SSM layer: conv -> SiLU -> projections -> scan -> gate, forward and backward
// with recomputation (see include/ss_layer.h).
//
// The scan, the convolution and the projections are all this library's own kernels (ss::gemm for
// the projections and their gradients).  Everything is laid out so that no product needs a
// transposed copy of a (B, D, L) tensor: with the sequence axis last, a batch entry of u is a
// (D, L) row-major matrix, [r;B;C] = W_x @ u lands directly in the (B, N, L) layout the scan reads
// (B and C are rows R.. of the result: the scan is told the batch stride), and
// delta_raw = W_dt @ r lands in the (B, D, L) layout of the scan's step-size input.
#include <hip/hip_runtime.h>

#include "ss_device.h"
#include "ss_kernels.h"
#include "ss_layer.h"

namespace {

inline bool aligned_to(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// C[i] (M x N) = op(A[i]) (M x K) @ op(B[i]) (K x N) + beta * C[i] (beta 0 or 1), all ROW-major with
// row pitches lda/ldb/ldc of the stored matrices and element strides sA/sB/sC between batch
// entries; C is float32 if c_float, else in the io dtype.
bool gemm_rm(hipStream_t st, bool tA, bool tB, int M, int N, int K, const void* A, int lda, long sA,
             const void* B, int ldb, long sB, float beta, void* C, int ldc, long sC, int batch, bool bf16, bool c_float = false,
             void* split_ws = nullptr, size_t split_ws_bytes = 0)
{
    ss::GemmArgs g{};
    g.M = M; g.N = N; g.K = K; g.batch = batch;
    g.A = A; g.a_m = tA ? 1 : lda; g.a_k = tA ? lda : 1; g.a_batch = sA;
    g.B = B; g.b_k = tB ? 1 : ldb; g.b_n = tB ? ldb : 1; g.b_batch = sB;
    g.C = C; g.ldc = ldc; g.c_batch = sC;
    g.bf16 = bf16; g.c_float = c_float || !bf16; g.accumulate = beta != 0.0f;
    g.split_ws = split_ws; g.split_ws_bytes = split_ws_bytes;
    return ss::gemm(g, st) == SS_OK;
}

// ---- small kernels around the GEMMs -----------------------------------------------------------
// dB, dC (B,N,L) float32 -> rows R.. of d[r;B;C] (B, R+2N, L) in the io dtype.
template <typename T>
__global__ void pack_dbc_kernel(const float* __restrict__ dB, const float* __restrict__ dC, T* __restrict__ dP,
                                int N, int R, long L, long total)
{
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;   // over B * 2N * L
    if (i >= total) return;
    const long l = i % L;
    const long row = i / L;               // b * 2N + j
    const long b = row / (2 * N);
    const int j = int(row - b * 2 * N);   // 0..N-1: B, N..2N-1: C
    const float v = j < N ? dB[(b * N + j) * L + l] : dC[(b * N + (j - N)) * L + l];
    T* dst = dP + (b * (R + 2 * N) + R + j) * L + l;
    if constexpr (sizeof(T) == 2) *dst = T(ss::f32_to_bf16_bits(v));
    else *dst = v;
}

// out[i] = sum_b part[b][i], float32 accumulation in batch order.
template <typename T>
__global__ void sum_partials_kernel(const T* __restrict__ part, int nb, long n, float* __restrict__ out)
{
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    float acc = 0.0f;
    for (int b = 0; b < nb; ++b) {
        if constexpr (sizeof(T) == 2) acc += ss::bf16_to_f32(part[b * n + i]);
        else acc += part[b * n + i];
    }
    out[i] = acc;
}

// ---- decode: [r;B;C]_t = u_t @ W_x^T on the matrix cores --------------------------------------------
// P (nb, nm) float32 = u (nb, D) @ W (nm, D)^T, both operands bf16 with the contraction index
// contiguous, which is exactly how v_mfma_f32_16x16x32_bf16 wants its fragments: lane l supplies row
// l % 16 of either operand and the 8 consecutive k starting at 8 * (l / 16), one 16-byte load each, no
// staging.  The product is tiny (64 x 160 x 4096 for the headline layer) and bound by the latency of
// getting W and u on chip, so it is spread thin: workgroup (x, y, z) owns the 16 x 16 tile (x, y) of P
// over the z-th part of the contraction index and spreads that part over its eight waves (k-steps of
// 32, four per wave); the waves' accumulators are added through LDS in a fixed order and written to
// the z-th partial result, P + z * nb * nm.  The consumer adds the few partial results, again in a
// fixed order, so the outcome does not depend on timing (atomics across workgroups would make it
// so).  Requires D % 32 == 0.
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
constexpr int XP_WAVES = 8;
constexpr int XP_NPARTS = ss::STEP_NPARTS;   // partial results (fixed, so that the consumer can unroll over them)

__global__ void __launch_bounds__(64 * XP_WAVES) xproj_decode_kernel(const ss::bf16_t* __restrict__ u,
                                                                     const ss::bf16_t* __restrict__ W,
                                                                     float* __restrict__ P, int nb, int nm, int D)
{
    __shared__ f32x4_t part[XP_WAVES - 1][64];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int row0 = blockIdx.x * 16, col0 = blockIdx.y * 16;   // tile of P; its columns are rows of W
    const int urow = min(row0 + (lane & 15), nb - 1);           // rows past the end shadow the last one
    const int wrow = min(col0 + (lane & 15), nm - 1);
    const int ksub = 8 * (lane >> 4);
    const ss::bf16_t* up = u + (size_t)urow * D + ksub;
    const ss::bf16_t* wp = W + (size_t)wrow * D + ksub;
    f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
    constexpr int STRIDE = 32 * XP_WAVES;
    const int kpart = ((D + XP_NPARTS - 1) / XP_NPARTS + 31) / 32 * 32;   // contraction elements per part
    const int kend = min(D, (int)(blockIdx.z + 1) * kpart);
    int k = blockIdx.z * kpart + 32 * wave;
    for (; k + 3 * STRIDE < kend; k += 4 * STRIDE) {   // four k-steps' loads in flight together
        bf16x8_t a[4], b[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            a[i] = *reinterpret_cast<const bf16x8_t*>(up + k + i * STRIDE);
            b[i] = *reinterpret_cast<const bf16x8_t*>(wp + k + i * STRIDE);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i], b[i], acc, 0, 0, 0);
    }
    for (; k < kend; k += STRIDE)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<const bf16x8_t*>(up + k),
                                                     *reinterpret_cast<const bf16x8_t*>(wp + k), acc, 0, 0, 0);
    if (wave > 0) part[wave - 1][lane] = acc;
    __syncthreads();
    if (wave == 0) {
#pragma unroll
        for (int w = 0; w < XP_WAVES - 1; ++w) acc += part[w][lane];
        // accumulator element r of lane l is row 4 * (l / 16) + r, column l % 16 of the tile
        const int col = col0 + (lane & 15);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = row0 + 4 * (lane >> 4) + r;
            if (row < nb && col < nm) P[((size_t)blockIdx.z * nb + row) * nm + col] = acc[r];
        }
    }
}

// r (the first R rows of each batch entry of P, (B, Mx, L)) transposed and zero-padded to
// (B, Lp, Rp), for the delta projection inside the scan kernel (see FwdArgs::rT).  32 x 32 tiles
// through LDS; block (32, 8), grid (Lp / 32, Rp / 32, B).
__global__ void transpose_r_kernel(const ss::bf16_t* __restrict__ P, long bstride, ss::bf16_t* __restrict__ rT, int R, int L,
                                   int Lp, int Rp)
{
    __shared__ ss::bf16_t tile[32][33];
    const int t0 = blockIdx.x * 32, r0 = blockIdx.y * 32, b = blockIdx.z;
    const int tx = threadIdx.x, ty = threadIdx.y;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = r0 + ty + 8 * i, t = t0 + tx;
        tile[ty + 8 * i][tx] = (r < R && t < L) ? P[(size_t)b * bstride + (size_t)r * L + t] : ss::bf16_t(0);
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int t = t0 + ty + 8 * i, r = r0 + tx;
        rT[((size_t)b * Lp + t) * Rp + r] = tile[tx][ty + 8 * i];
    }
}

// dst (cols, rows) = src (rows, cols)^T for a weight matrix, 32 x 32 tiles through LDS; block (32, 8),
// grid (cols / 32 rounded up, rows / 32 rounded up).
template <typename T>
__global__ void transpose_weight_kernel(const T* __restrict__ src, T* __restrict__ dst, int rows, int cols)
{
    __shared__ T tile[32][33];
    const int c0 = blockIdx.x * 32, r0 = blockIdx.y * 32;
    const int tx = threadIdx.x, ty = threadIdx.y;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = r0 + ty + 8 * i, c = c0 + tx;
        if (r < rows && c < cols) tile[ty + 8 * i][tx] = src[(size_t)r * cols + c];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int c = c0 + ty + 8 * i, r = r0 + tx;
        if (r < rows && c < cols) dst[(size_t)c * rows + r] = tile[tx][ty + 8 * i];
    }
}
template <typename T>
bool transpose_weight(const void* src, void* dst, int rows, int cols, hipStream_t st)
{
    hipLaunchKernelGGL(transpose_weight_kernel<T>, dim3((unsigned)((cols + 31) / 32), (unsigned)((rows + 31) / 32)), dim3(32, 8), 0, st,
                       static_cast<const T*>(src), static_cast<T*>(dst), rows, cols);
    return hipGetLastError() == hipSuccess;
}

// ---- buffers -------------------------------------------------------------------------------------
struct Shape {
    size_t B, D, L, N, R, Mx, esz;
};
Shape shape_of(const ss_layer_params* p)
{
    Shape s;
    s.B = p->batch; s.D = p->dim; s.L = p->seqlen; s.N = p->dstate; s.R = p->dt_rank;
    s.Mx = s.R + 2 * s.N;
    s.esz = p->io_dtype == SS_BF16 ? 2 : 4;
    return s;
}

ss_fwd_params scan_params(const ss_layer_params* p)
{
    ss_fwd_params f{};
    f.batch = p->batch; f.dim = p->dim; f.seqlen = p->seqlen; f.dstate = p->dstate;
    f.io_dtype = p->io_dtype;
    f.flags = SS_DELTA_SOFTPLUS | SS_HAS_DELTA_BIAS | SS_HAS_D | SS_HAS_Z;
    return f;
}

// saved:   [P = [r;B;C] (B, Mx, L) io][workspace of the scan]
struct SavedLayout { size_t P_off, scan_off, scan_bytes, total; };
SavedLayout saved_layout(const ss_layer_params* p)
{
    const Shape s = shape_of(p);
    const ss_fwd_params f = scan_params(p);
    SavedLayout w{};
    w.P_off = 0;
    w.scan_off = round_up(s.B * s.Mx * s.L * s.esz, 256);
    w.scan_bytes = ss_workspace_bytes(&f, 1);
    w.total = w.scan_off + round_up(w.scan_bytes, 256);
    return w;
}

// scratch: forward  [u][delta][P and the scan's split scratch, used if nothing is saved][r transposed and padded, bf16]
//          backward [u][delta][du][ddelta][dP (B,Mx,L) io][dB, dC (B,N,L) f32]
//                   [partials of dW_dt (B,D,R) f32][partials of dW_x (B,Mx,D) f32]
//                   [W_dt transposed (R,D) io][W_x transposed (D,Mx) io]
//          both     [float32 shares of a projection whose contraction is split across workgroups (B,Mx,L) x 2]
struct ScratchLayout { size_t u, delta, P, scan_ws, scan_ws_bytes, rT, du, ddelta, dP, dB, dC, part_dt, part_x, WdtT, WxT, gsplit, gsplit_bytes, total; };
ScratchLayout scratch_layout(const ss_layer_params* p, bool bwd)
{
    const Shape s = shape_of(p);
    ScratchLayout w{};
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t at = off; off += round_up(bytes, 256); return at; };
    // The (B,D,L) buffers start 65 KiB (a multiple of 256 bytes) further apart than their size: the scan
    // touches all of them at the same row and step, and with rows a large power of two of bytes apart equal
    // starting offsets into the memory channels' interleave would put all of that on one channel.
    constexpr size_t SKEW = 66560;
    const size_t T = s.B * s.D * s.L * s.esz + SKEW;
    w.u = take(T);
    w.delta = take(T);
    if (!bwd) {
        w.P = take(s.B * s.Mx * s.L * s.esz);
        const ss_fwd_params f = scan_params(p);
        w.scan_ws_bytes = ss_workspace_bytes(&f, 0);
        w.scan_ws = take(w.scan_ws_bytes);
        w.rT = take(s.B * round_up(s.L, 32) * round_up(s.R, 32) * s.esz);
    } else {
        w.du = take(T);
        w.ddelta = take(T);
        w.dP = take(s.B * s.Mx * s.L * s.esz);
        w.dB = take(s.B * s.N * s.L * sizeof(float));
        w.dC = take(s.B * s.N * s.L * sizeof(float));
        w.part_dt = take(s.B * s.D * s.R * sizeof(float));
        w.part_x = take(s.B * s.Mx * s.D * sizeof(float));
        w.WdtT = take(s.R * s.D * s.esz);
        w.WxT = take(s.D * s.Mx * s.esz);
    }
    w.gsplit_bytes = 2 * s.B * s.Mx * s.L * sizeof(float);
    w.gsplit = take(w.gsplit_bytes);
    w.total = off;
    return w;
}

bool shape_ok(const ss_layer_params* p)
{
    return p->batch >= 1 && p->dim >= 1 && p->seqlen >= 1 && p->dstate >= 1 && p->dt_rank >= 1 && p->conv_width >= 1;
}

int check_layer(const ss_layer_params* p, bool bwd)
{
    if (!p) return SS_ERR_NULL;
    if (!shape_ok(p)) return SS_ERR_SHAPE;
    if (p->dstate > SS_MAX_DSTATE || p->conv_width > SS_CONV_MAX_WIDTH) return SS_ERR_UNSUPPORTED;
    if (p->io_dtype != SS_F32 && p->io_dtype != SS_BF16) return SS_ERR_UNSUPPORTED;
    if (p->flags != 0) return SS_ERR_UNSUPPORTED;
    // the projections take 32-bit sizes
    if ((long)p->dim * p->dt_rank >= 0x7fffffffL || (long)p->dim * (p->dt_rank + 2 * p->dstate) >= 0x7fffffffL)
        return SS_ERR_UNSUPPORTED;
    if (!p->x || !p->z || !p->conv_w || !p->conv_b || !p->W_x || !p->W_dt || !p->dt_bias || !p->A || !p->Dskip)
        return SS_ERR_NULL;
    if (!bwd && !p->out) return SS_ERR_NULL;
    if (!bwd && ((p->h_last && !aligned_to(p->h_last, 4)) || (p->conv_state && !aligned_to(p->conv_state, 2))))
        return SS_ERR_ALIGN;
    const void* io[] = {p->x, p->z, p->W_x, p->W_dt, bwd ? nullptr : p->out};
    for (const void* q : io)
        if (q && !aligned_to(q, 16)) return SS_ERR_ALIGN;
    const void* f32[] = {p->conv_w, p->conv_b, p->dt_bias, p->A, p->Dskip};
    for (const void* q : f32)
        if (!aligned_to(q, 4)) return SS_ERR_ALIGN;
    if (bwd || p->saved) {
        if (!p->saved || p->saved_bytes < saved_layout(p).total) return SS_ERR_WORKSPACE;
        if (!aligned_to(p->saved, 256)) return SS_ERR_ALIGN;
    }
    if (!p->scratch || p->scratch_bytes < scratch_layout(p, bwd).total) return SS_ERR_WORKSPACE;
    if (!aligned_to(p->scratch, 256)) return SS_ERR_ALIGN;
    return SS_OK;
}

ss_conv_params conv_params(const ss_layer_params* p, void* u)
{
    ss_conv_params c{};
    c.batch = p->batch; c.dim = p->dim; c.seqlen = p->seqlen; c.width = p->conv_width;
    c.io_dtype = p->io_dtype;
    c.flags = SS_CONV_SILU | SS_CONV_HAS_BIAS;
    c.x = p->x; c.w = p->conv_w; c.bias = p->conv_b;
    c.out = u;
    return c;
}

}  // namespace

extern "C" {

size_t ss_layer_saved_bytes(const ss_layer_params* p)
{
    if (!p || !shape_ok(p)) return 0;
    return saved_layout(p).total;
}

size_t ss_layer_scratch_bytes(const ss_layer_params* p, int for_backward)
{
    if (!p || !shape_ok(p)) return 0;
    return scratch_layout(p, for_backward != 0).total;
}

int ss_layer_fwd(const ss_layer_params* p, void* stream)
{
    int rc = check_layer(p, false);
    if (rc != SS_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const Shape s = shape_of(p);
    const bool bf16 = p->io_dtype == SS_BF16;
    const ScratchLayout sc = scratch_layout(p, false);
    const SavedLayout sv = saved_layout(p);
    char* scratch = static_cast<char*>(p->scratch);
    char* saved = static_cast<char*>(p->saved);
    char* u = scratch + sc.u;
    char* delta = scratch + sc.delta;
    char* P = saved ? saved + sv.P_off : scratch + sc.P;
    const int B = p->batch, D = p->dim, L = p->seqlen, N = p->dstate, R = p->dt_rank, Mx = R + 2 * N;

    ss_conv_params c = conv_params(p, u);
    if (p->conv_state && p->conv_width > 1) {
        c.flags |= SS_CONV_WRITE_STATE;
        c.state_out = p->conv_state;
    }
    if ((rc = ss_conv_fwd(&c, stream)) != SS_OK) return rc;
    // [r;B;C] = W_x @ u
    if (!gemm_rm(st, false, false, Mx, L, D, p->W_x, D, 0, u, L, (long)D * L, 0.0f, P, L, (long)Mx * L, B, bf16, false,
                 scratch + sc.gsplit, sc.gsplit_bytes))
        return SS_ERR_LAUNCH;
    ss_fwd_params f = scan_params(p);
    f.u = u; f.delta = delta; f.z = p->z;
    f.Bmat = P + (size_t)R * L * s.esz;
    f.Cmat = P + (size_t)(R + N) * L * s.esz;
    f.A = p->A; f.Dskip = p->Dskip; f.delta_bias = p->dt_bias;
    f.out = p->out;
    if (p->h_last) {
        f.flags |= SS_WRITE_H_LAST;
        f.h_last = p->h_last;
    }
    if (saved) {
        f.flags |= SS_SAVE_FOR_BWD;
        f.workspace = saved + sv.scan_off;
        f.workspace_bytes = sv.scan_bytes;
    } else if (sc.scan_ws_bytes) {
        f.workspace = scratch + sc.scan_ws;   // lets a long sequence with few rows be split
        f.workspace_bytes = sc.scan_ws_bytes;
    }
    // bf16: delta_raw = W_dt r is formed inside the scan kernel where that variant applies
    if (ss::scan_fwd_fusable(&f, R)) {
        ss::bf16_t* rT = reinterpret_cast<ss::bf16_t*>(scratch + sc.rT);
        const int Lp = (L + 31) / 32 * 32, Rp = (R + 31) / 32 * 32;
        hipLaunchKernelGGL(transpose_r_kernel, dim3((unsigned)(Lp / 32), (unsigned)(Rp / 32), (unsigned)B), dim3(32, 8), 0, st,
                           reinterpret_cast<const ss::bf16_t*>(P), (long)Mx * L, rT, R, L, Lp, Rp);
        if (hipGetLastError() != hipSuccess) return SS_ERR_LAUNCH;
        rc = ss::scan_fwd_fused(&f, (long)Mx * L, p->W_dt, R, rT, stream);
        if (rc != SS_ERR_UNSUPPORTED) return rc;   // otherwise nothing was enqueued: take the general path
    }
    // delta_raw = W_dt @ r
    if (!gemm_rm(st, false, false, D, L, R, p->W_dt, R, 0, P, L, (long)Mx * L, 0.0f, delta, L, (long)D * L, B, bf16))
        return SS_ERR_LAUNCH;
    return ss::scan_fwd_strided(&f, (long)Mx * L, stream);
}

int ss_layer_bwd(const ss_layer_bwd_params* q, void* stream)
{
    if (!q) return SS_ERR_NULL;
    const ss_layer_params* p = &q->fwd;
    int rc = check_layer(p, true);
    if (rc != SS_OK) return rc;
    if (!q->dout || !q->dx || !q->dz || !q->dconv_w || !q->dconv_b || !q->dW_x || !q->dW_dt || !q->ddt_bias ||
        !q->dA || !q->dD)
        return SS_ERR_NULL;
    if (!aligned_to(q->dout, 16) || !aligned_to(q->dx, 16) || !aligned_to(q->dz, 16)) return SS_ERR_ALIGN;
    const void* f32[] = {q->dconv_w, q->dconv_b, q->dW_x, q->dW_dt, q->ddt_bias, q->dA, q->dD};
    for (const void* g : f32)
        if (!aligned_to(g, 4)) return SS_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const Shape s = shape_of(p);
    const bool bf16 = p->io_dtype == SS_BF16;
    const ScratchLayout sc = scratch_layout(p, true);
    const SavedLayout sv = saved_layout(p);
    char* scratch = static_cast<char*>(p->scratch);
    char* saved = static_cast<char*>(p->saved);
    char *u = scratch + sc.u, *delta = scratch + sc.delta, *du = scratch + sc.du, *ddelta = scratch + sc.ddelta;
    char *dP = scratch + sc.dP, *part_dt = scratch + sc.part_dt, *part_x = scratch + sc.part_x;
    float* dB = reinterpret_cast<float*>(scratch + sc.dB);
    float* dC = reinterpret_cast<float*>(scratch + sc.dC);
    char* P = saved + sv.P_off;
    const int B = p->batch, D = p->dim, L = p->seqlen, N = p->dstate, R = p->dt_rank, Mx = R + 2 * N;

    // recompute the two cheap intermediates
    ss_conv_params c = conv_params(p, u);
    if ((rc = ss_conv_fwd(&c, stream)) != SS_OK) return rc;
    if (!gemm_rm(st, false, false, D, L, R, p->W_dt, R, 0, P, L, (long)Mx * L, 0.0f, delta, L, (long)D * L, B, bf16))
        return SS_ERR_LAUNCH;

    // the scan
    ss_bwd_params b{};
    b.fwd = scan_params(p);
    b.fwd.u = u; b.fwd.delta = delta; b.fwd.z = p->z;
    b.fwd.Bmat = P + (size_t)R * L * s.esz;
    b.fwd.Cmat = P + (size_t)(R + N) * L * s.esz;
    b.fwd.A = p->A; b.fwd.Dskip = p->Dskip; b.fwd.delta_bias = p->dt_bias;
    b.fwd.workspace = saved + sv.scan_off;
    b.fwd.workspace_bytes = sv.scan_bytes;
    b.dout = q->dout;
    b.du = du; b.ddelta = ddelta; b.dz = q->dz;
    b.dB = dB; b.dC = dC;
    b.dA = q->dA; b.dD = q->dD; b.ddelta_bias = q->ddt_bias;
    if ((rc = ss::scan_bwd_strided(&b, (long)Mx * L, stream)) != SS_OK) return rc;

    // The two products with a transposed weight take it from a transposed copy (a megabyte each), so
    // that their first operand is contiguous along the contraction index like everywhere else.
    char *WdtT = scratch + sc.WdtT, *WxT = scratch + sc.WxT;
    if (!(bf16 ? transpose_weight<ss::bf16_t>(p->W_dt, WdtT, D, R, st) : transpose_weight<float>(p->W_dt, WdtT, D, R, st)) ||
        !(bf16 ? transpose_weight<ss::bf16_t>(p->W_x, WxT, Mx, D, st) : transpose_weight<float>(p->W_x, WxT, Mx, D, st)))
        return SS_ERR_LAUNCH;
    // delta_raw = W_dt @ r:  dr = W_dt^T @ ddelta  (rows 0..R-1 of dP),  dW_dt = sum_b ddelta r^T
    if (!gemm_rm(st, false, false, R, L, D, WdtT, D, 0, ddelta, L, (long)D * L, 0.0f, dP, L, (long)Mx * L, B, bf16, false,
                 scratch + sc.gsplit, sc.gsplit_bytes))
        return SS_ERR_LAUNCH;
    if (!gemm_rm(st, false, true, D, R, L, ddelta, L, (long)D * L, P, L, (long)Mx * L, 0.0f, part_dt, R, (long)D * R, B, bf16, true))
        return SS_ERR_LAUNCH;
    // rows R.. of dP from the scan's float32 dB, dC
    {
        const long total = (long)B * 2 * N * L;
        const dim3 grid((unsigned)((total + 255) / 256));
        if (bf16) hipLaunchKernelGGL(pack_dbc_kernel<ss::bf16_t>, grid, dim3(256), 0, st, dB, dC, reinterpret_cast<ss::bf16_t*>(dP), N, R, (long)L, total);
        else hipLaunchKernelGGL(pack_dbc_kernel<float>, grid, dim3(256), 0, st, dB, dC, reinterpret_cast<float*>(dP), N, R, (long)L, total);
        if (hipGetLastError() != hipSuccess) return SS_ERR_LAUNCH;
    }
    // [r;B;C] = W_x @ u:  du += W_x^T @ dP,  dW_x = sum_b dP u^T
    if (!gemm_rm(st, false, false, D, L, Mx, WxT, Mx, 0, dP, L, (long)Mx * L, 1.0f, du, L, (long)D * L, B, bf16))
        return SS_ERR_LAUNCH;
    if (!gemm_rm(st, false, true, Mx, D, L, dP, L, (long)Mx * L, u, L, (long)D * L, 0.0f, part_x, D, (long)Mx * D, B, bf16, true))
        return SS_ERR_LAUNCH;
    {
        const long n_dt = (long)D * R, n_x = (long)Mx * D;
        hipLaunchKernelGGL(sum_partials_kernel<float>, dim3((unsigned)((n_dt + 255) / 256)), dim3(256), 0, st, reinterpret_cast<const float*>(part_dt), B, n_dt, q->dW_dt);
        hipLaunchKernelGGL(sum_partials_kernel<float>, dim3((unsigned)((n_x + 255) / 256)), dim3(256), 0, st, reinterpret_cast<const float*>(part_x), B, n_x, q->dW_x);
        if (hipGetLastError() != hipSuccess) return SS_ERR_LAUNCH;
    }
    // u = SiLU(conv(x))
    ss_conv_bwd_params cb{};
    cb.fwd = conv_params(p, nullptr);
    cb.dout = du; cb.dx = q->dx; cb.dw = q->dconv_w; cb.dbias = q->dconv_b;
    return ss_conv_bwd(&cb, stream);
}

size_t ss_layer_step_scratch_bytes(const ss_layer_step_params* p)
{
    if (!p || p->batch < 1 || p->dim < 1 || p->dstate < 1 || p->dt_rank < 1) return 0;
    const size_t esz = p->io_dtype == SS_BF16 ? 2 : 4;
    const size_t B = p->batch, D = p->dim, Mx = (size_t)p->dt_rank + 2 * (size_t)p->dstate;
    // u_t, delta_t, [r;B;C]_t in the io dtype, and the float32 partial results of the bf16 path's projection
    return 2 * round_up(B * D * esz, 256) + round_up(B * Mx * esz, 256) + round_up(XP_NPARTS * B * Mx * sizeof(float), 256);
}

int ss_layer_step(const ss_layer_step_params* p, void* stream)
{
    if (!p) return SS_ERR_NULL;
    if (p->batch < 1 || p->dim < 1 || p->dstate < 1 || p->dt_rank < 1 || p->conv_width < 1) return SS_ERR_SHAPE;
    if (p->dstate > SS_MAX_DSTATE || p->conv_width > SS_CONV_MAX_WIDTH) return SS_ERR_UNSUPPORTED;
    if (p->io_dtype != SS_F32 && p->io_dtype != SS_BF16) return SS_ERR_UNSUPPORTED;
    if (p->flags != 0) return SS_ERR_UNSUPPORTED;
    if (!p->h || !p->x_t || !p->z_t || !p->conv_w || !p->conv_b || !p->W_x || !p->W_dt || !p->dt_bias || !p->A ||
        !p->Dskip || !p->out_t || (p->conv_width > 1 && !p->conv_state))
        return SS_ERR_NULL;
    if (!aligned_to(p->W_x, 16) || !aligned_to(p->W_dt, 16)) return SS_ERR_ALIGN;
    if (!p->scratch || p->scratch_bytes < ss_layer_step_scratch_bytes(p)) return SS_ERR_WORKSPACE;
    if (!aligned_to(p->scratch, 256)) return SS_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool bf16 = p->io_dtype == SS_BF16;
    const size_t esz = bf16 ? 2 : 4;
    const int B = p->batch, D = p->dim, N = p->dstate, R = p->dt_rank, Mx = R + 2 * N;
    char* scratch = static_cast<char*>(p->scratch);
    char* u_t = scratch;
    char* delta_t = u_t + round_up((size_t)B * D * esz, 256);
    char* P_t = delta_t + round_up((size_t)B * D * esz, 256);

    float* P_acc = reinterpret_cast<float*>(P_t + round_up((size_t)B * Mx * esz, 256));

    ss_conv_step_params c{};
    c.batch = B; c.dim = D; c.width = p->conv_width; c.io_dtype = p->io_dtype;
    c.flags = SS_CONV_SILU | SS_CONV_HAS_BIAS;
    c.state = p->conv_state; c.x_t = p->x_t; c.w = p->conv_w; c.bias = p->conv_b; c.out_t = u_t;
    ss_step_params s{};
    s.batch = B; s.dim = D; s.dstate = N; s.io_dtype = p->io_dtype;
    s.flags = SS_DELTA_SOFTPLUS | SS_HAS_DELTA_BIAS | SS_HAS_D | SS_HAS_Z;
    s.h = p->h; s.u_t = u_t; s.z_t = p->z_t;
    s.A = p->A; s.Dskip = p->Dskip; s.delta_bias = p->dt_bias;
    s.out_t = p->out_t;

    // bf16 with friendly sizes: both projections on the matrix cores, delta_t = W_dt r_t inside the
    // state-update kernel -- three launches, no library call, no atomics
    auto aligned16 = [](const void* q) { return reinterpret_cast<uintptr_t>(q) % 16 == 0; };
    if (bf16 && D % 32 == 0 && R % 8 == 0 && R <= 256 && N <= 16 && Mx % 4 == 0 && aligned16(p->W_x) && aligned16(p->W_dt) &&
        aligned16(p->h)) {
        int rc = ss_conv_step(&c, stream);
        if (rc != SS_OK) return rc;
        const dim3 grid((unsigned)((B + 15) / 16), (unsigned)((Mx + 15) / 16), (unsigned)XP_NPARTS);
        hipLaunchKernelGGL(xproj_decode_kernel, grid, dim3(64 * XP_WAVES), 0, st, reinterpret_cast<const ss::bf16_t*>(u_t),
                           static_cast<const ss::bf16_t*>(p->W_x), P_acc, B, Mx, D);
        if (hipGetLastError() != hipSuccess) return SS_ERR_LAUNCH;
        return ss::step_projected(&s, P_acc, p->W_dt, R, Mx, stream);
    }

    int rc = ss_conv_step(&c, stream);
    if (rc != SS_OK) return rc;
    // [r;B;C]_t (B, Mx) = u_t (B, D) @ W_x^T;   delta_t (B, D) = r_t (B, R) @ W_dt^T
    if (!gemm_rm(st, false, true, B, Mx, D, u_t, D, 0, p->W_x, D, 0, 0.0f, P_t, Mx, 0, 1, bf16)) return SS_ERR_LAUNCH;
    if (!gemm_rm(st, false, true, B, D, R, P_t, Mx, 0, p->W_dt, R, 0, 0.0f, delta_t, D, 0, 1, bf16)) return SS_ERR_LAUNCH;
    s.delta_t = delta_t;
    s.B_t = P_t + (size_t)R * esz;
    s.C_t = P_t + (size_t)(R + N) * esz;
    return ss::step_strided(&s, Mx, stream);
}

int ss_proj_gemm(const ss_gemm_params* p, void* stream)
{
    if (!p) return SS_ERR_NULL;
    if (p->M < 0 || p->N < 0 || p->K < 0 || p->batch < 0) return SS_ERR_SHAPE;
    if (p->io_dtype != SS_F32 && p->io_dtype != SS_BF16) return SS_ERR_UNSUPPORTED;
    if (p->flags & ~(SS_GEMM_C_FLOAT | SS_GEMM_ACCUMULATE | SS_GEMM_GENERAL)) return SS_ERR_UNSUPPORTED;
    if (p->M == 0 || p->N == 0 || p->batch == 0) return SS_OK;
    if (!p->C || (p->K > 0 && (!p->A || !p->B))) return SS_ERR_NULL;   // K = 0: an empty sum, A and B are not read
    ss::GemmArgs g{};
    g.M = p->M; g.N = p->N; g.K = p->K; g.batch = p->batch;
    g.A = p->A; g.a_m = p->a_m; g.a_k = p->a_k; g.a_batch = p->a_batch;
    g.B = p->B; g.b_k = p->b_k; g.b_n = p->b_n; g.b_batch = p->b_batch;
    g.C = p->C; g.ldc = p->ldc; g.c_batch = p->c_batch;
    g.bf16 = p->io_dtype == SS_BF16;
    g.c_float = (p->flags & SS_GEMM_C_FLOAT) || !g.bf16;
    g.accumulate = p->flags & SS_GEMM_ACCUMULATE;
    g.general = p->flags & SS_GEMM_GENERAL;
    if (p->workspace && aligned_to(p->workspace, 256)) {
        g.split_ws = p->workspace;
        g.split_ws_bytes = p->workspace_bytes;
    }
    return ss::gemm(g, static_cast<hipStream_t>(stream));
}

size_t ss_proj_gemm_workspace_bytes(const ss_gemm_params* p)
{
    if (!p || p->M < 0 || p->N < 0 || p->batch < 0) return 0;
    return 2 * (size_t)p->batch * (size_t)p->M * (size_t)p->N * sizeof(float);
}

}  // extern "C"
