// Short causal per-channel convolution (+ SiLU): forward, backward and single-token step
// for gfx950, with their C-ABI entry points (see include/ss_conv.h).
//
// The operation moves 2-3 tensors of (B,D,L) elements and does about ten flops per
// element, so it is bound by HBM and the kernels are organised around 16-byte accesses:
// a lane owns 8 consecutive steps of one (b,d) row, a wave owns a "piece" of 512 steps.
// The W-1 samples in front of a lane's slice are fetched with one extra 8- or 16-byte load
// that hits the line the neighbouring lane has just brought in.  Taps are kept
// right-aligned in four slots (slot j multiplies x[t-3+j]; unused leading slots are zero),
// so one code path serves every width up to 4.
#include <hip/hip_runtime.h>

#include "ss_conv.h"
#include "ss_device.h"

namespace ss {

constexpr int TAPS = SS_CONV_MAX_WIDTH;  // 4
constexpr int HALO = TAPS - 1;           // 3
constexpr int PIECE = WAVE * 8;          // steps one wave covers per pass

struct ConvArgs {
    int B, D, L, W;
    unsigned flags;
    const void *x, *state_in, *dout;
    const float *w, *bias;
    void *out, *state_out, *dx;
    float *dw, *dbias;
};

template <typename T> __device__ __forceinline__ float io_to_f32(T v);
template <> __device__ __forceinline__ float io_to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float io_to_f32<bf16_t>(bf16_t v) { return bf16_to_f32(v); }
template <typename T> __device__ __forceinline__ T f32_to_io(float v);
template <> __device__ __forceinline__ float f32_to_io<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t f32_to_io<bf16_t>(float v) { return bf16_t(f32_to_bf16_bits(v)); }

__device__ __forceinline__ void load_taps(const float* __restrict__ w, int d, int W, float (&k4)[TAPS])
{
#pragma unroll
    for (int j = 0; j < TAPS; ++j) {
        const int k = j - (TAPS - W);
        k4[j] = k >= 0 ? w[(size_t)d * W + k] : 0.0f;
    }
}

// Sample of the sequence before its start: index t in [-(W-1), -1] comes from state_in.
template <typename T>
__device__ __forceinline__ float before_start(const T* __restrict__ state_row, int t, int W)
{
    const int idx = t + (W - 1);
    return (state_row != nullptr && idx >= 0) ? io_to_f32<T>(state_row[idx]) : 0.0f;
}

// xs[0..2] = x[t0-3..t0-1], xs[3..10] = x[t0..t0+7] (zero past the end of the row).
template <typename T, bool VEC>
__device__ __forceinline__ void load_window(const T* __restrict__ row, const T* __restrict__ state_row, int t0,
                                            int L, int W, float (&xs)[HALO + 8])
{
    const int nvalid = min(max(L - t0, 0), 8);
    float cur[8];
    io8<T>::unpack(io8<T>::template load<VEC>(row + t0, nvalid), cur);
#pragma unroll
    for (int j = 0; j < 8; ++j) xs[HALO + j] = cur[j];
    if (VEC && t0 > 0 && nvalid > 0) {
        // t0 is a multiple of 8, so the four samples in front of the slice are aligned
        float h[4];
        io4<T>::unpack(io4<T>::template load<true>(row + t0 - 4, 4), h);
        xs[0] = h[1]; xs[1] = h[2]; xs[2] = h[3];
    } else {
#pragma unroll
        for (int j = 0; j < HALO; ++j) {
            const int t = t0 - HALO + j;
            xs[j] = (nvalid == 0) ? 0.0f : (t >= 0 ? io_to_f32<T>(row[t]) : before_start<T>(state_row, t, W));
        }
    }
}

// The same for rows of whole 8-step slices (L a multiple of 8), in two halves so that all the
// loads of a unit are issued back to back and waited for once: branch-free buffer loads (an
// offset out of range returns zeros), where the pointer form above waits for each conditional
// load in turn.  `next` additionally fetches the 4 samples after the slice.
template <typename T>
struct window_raw {
    typename io8<T>::raw cur;
    typename io4<T>::raw halo, next;
    uint32_t st[HALO];
};
template <typename T>
__device__ __forceinline__ uint32_t row_bytes(int L) { return (uint32_t)L * (uint32_t)sizeof(T); }   // rows below 2^31 bytes (checked by the host)
template <typename T, bool NEXT>
__device__ __forceinline__ window_raw<T> issue_window(rsrc_t brow, rsrc_t bstate, int t0, int L, int W)
{
    window_raw<T> r;
    const uint32_t esz = (uint32_t)sizeof(T);
    r.cur = io8<T>::load_buf(brow, t0 < L ? (uint32_t)t0 * esz : BUF_OFF);
    // t0 is a multiple of 8, so the four samples in front of the slice are aligned
    r.halo = io4<T>::load_buf(brow, (t0 > 0 && t0 < L) ? (uint32_t)(t0 - 4) * esz : BUF_OFF);
    if (NEXT) r.next = io4<T>::load_buf(brow, t0 + 8 < L ? (uint32_t)(t0 + 8) * esz : BUF_OFF);
#pragma unroll
    for (int j = 0; j < HALO; ++j) {   // the window handed over from before the sequence, for the row's first slice
        const int idx = j - (TAPS - W);
        r.st[j] = buf_load_elem<T>(bstate, (t0 == 0 && idx >= 0) ? (uint32_t)idx * esz : BUF_OFF);
    }
    return r;
}
template <typename T>
__device__ __forceinline__ float raw_to_f32(uint32_t bits)
{
    if constexpr (sizeof(T) == 2) return bf16_to_f32(bf16_t(bits)); else return __uint_as_float(bits);
}
// xs as load_window; xn[0..3] = x[t0+8..t0+11] if fetched
template <typename T, bool NEXT>
__device__ __forceinline__ void unpack_window(const window_raw<T>& r, int t0, float (&xs)[HALO + 8], float (&xn)[4])
{
    float cur[8], h[4];
    io8<T>::unpack(r.cur, cur);
    io4<T>::unpack(r.halo, h);
#pragma unroll
    for (int j = 0; j < 8; ++j) xs[HALO + j] = cur[j];
#pragma unroll
    for (int j = 0; j < HALO; ++j) xs[j] = t0 > 0 ? h[j + 1] : raw_to_f32<T>(r.st[j]);
    if (NEXT) io4<T>::unpack(r.next, xn);
}

__device__ __forceinline__ float conv_at(const float (&k4)[TAPS], float bias, const float* xs)
{
    return fmaf(k4[3], xs[3], fmaf(k4[2], xs[2], fmaf(k4[1], xs[1], fmaf(k4[0], xs[0], bias))));
}

// ---- forward --------------------------------------------------------------------------------
// One wave per (row, piece); grid = ceil(B*D*pieces / NWAVES) workgroups.
template <typename T, bool VEC, bool SILU>
__global__ __launch_bounds__(THREADS) void conv_fwd_kernel(const ConvArgs a)
{
    const int lane = threadIdx.x & (WAVE - 1);
    const int pieces = (a.L + PIECE - 1) / PIECE;
    const long unit = (long)blockIdx.x * NWAVES + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (unit >= (long)a.B * a.D * pieces) return;
    const long r = unit / pieces;                 // row b*D + d
    const int piece = int(unit - r * pieces);
    const int d = int(r % a.D);
    const int t0 = piece * PIECE + lane * 8;
    if (t0 >= a.L) return;

    const T* row = static_cast<const T*>(a.x) + (size_t)r * a.L;
    const T* state_row = (a.flags & SS_CONV_HAS_STATE) ? static_cast<const T*>(a.state_in) + (size_t)r * (a.W - 1) : nullptr;
    float k4[TAPS];
    load_taps(a.w, d, a.W, k4);
    const float bias = (a.flags & SS_CONV_HAS_BIAS) ? a.bias[d] : 0.0f;

    float xs[HALO + 8];
    if constexpr (VEC) {
        const rsrc_t brow = make_rsrc(row, row_bytes<T>(a.L));
        const rsrc_t bstate = make_rsrc(state_row ? state_row : row, state_row ? (uint32_t)(a.W - 1) * (uint32_t)sizeof(T) : 0u);
        float unused[4];
        unpack_window<T, false>(issue_window<T, false>(brow, bstate, t0, a.L, a.W), t0, xs, unused);
    } else {
        load_window<T, VEC>(row, state_row, t0, a.L, a.W, xs);
    }
    float o[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const float v = conv_at(k4, bias, xs + j);
        o[j] = SILU ? v * sigmoid_fast(v) : v;
    }
    const int nvalid = min(a.L - t0, 8);
    io8<T>::template store<VEC>(static_cast<T*>(a.out) + (size_t)r * a.L + t0, o, nvalid);

    if ((a.flags & SS_CONV_WRITE_STATE) && t0 + 8 >= a.L) {  // the lane that holds the last sample
        T* so = static_cast<T*>(a.state_out) + (size_t)r * (a.W - 1);
        for (int j = 0; j < a.W - 1; ++j) {
            const int i = a.L - (a.W - 1) + j - (t0 - HALO);    // position in xs, 0..10
            float v = 0.0f;
#pragma unroll
            for (int q = 0; q < HALO + 8; ++q) v = (q == i) ? xs[q] : v;
            so[j] = f32_to_io<T>(v);
        }
    }
}

// seqlen == 0: the window does not move.
template <typename T>
__global__ void conv_state_copy_kernel(const T* __restrict__ in, T* __restrict__ out, size_t n)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = in ? in[i] : T(0);
}

// ---- backward -------------------------------------------------------------------------------
// dx[t] = sum_j k4[j] * dv[t+3-j], dv = dout * SiLU'(v);  dk4[j] = sum_{b,t} dv[t] x[t-3+j].
// grid = (D, nsplit): the waves of column d share out its B*pieces (row, piece) units, keep
// the tap and bias gradients in registers and add them to dw/dbias once at the end.
template <typename T, bool VEC, bool SILU>
__global__ __launch_bounds__(THREADS) void conv_bwd_kernel(const ConvArgs a)
{
    const int lane = threadIdx.x & (WAVE - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int d = blockIdx.x;
    const int pieces = (a.L + PIECE - 1) / PIECE;
    const int units = a.B * pieces;
    const int stride = gridDim.y * NWAVES;

    float k4[TAPS];
    load_taps(a.w, d, a.W, k4);
    const float bias = (a.flags & SS_CONV_HAS_BIAS) ? a.bias[d] : 0.0f;
    float gk[TAPS] = {0.f, 0.f, 0.f, 0.f}, gb = 0.0f;

    for (int unit = blockIdx.y * NWAVES + wave; unit < units; unit += stride) {
        const int b = unit / pieces, piece = unit - b * pieces;
        const size_t r = (size_t)b * a.D + d;
        const int t0 = piece * PIECE + lane * 8;
        const T* row = static_cast<const T*>(a.x) + r * a.L;
        const T* grow = static_cast<const T*>(a.dout) + r * a.L;
        const T* state_row = (a.flags & SS_CONV_HAS_STATE) ? static_cast<const T*>(a.state_in) + r * (a.W - 1) : nullptr;
        const int nvalid = min(max(a.L - t0, 0), 8);

        float xs[HALO + 8], g[8], dv[8 + HALO];
        float xn[4] = {0.f, 0.f, 0.f, 0.f}, gn[4] = {0.f, 0.f, 0.f, 0.f};   // VEC: x and dout of the 4 steps after the slice
        if constexpr (VEC) {
            const rsrc_t brow = make_rsrc(row, row_bytes<T>(a.L));
            const rsrc_t bgrow = make_rsrc(grow, row_bytes<T>(a.L));
            const rsrc_t bstate = make_rsrc(state_row ? state_row : row, state_row ? (uint32_t)(a.W - 1) * (uint32_t)sizeof(T) : 0u);
            const uint32_t esz = (uint32_t)sizeof(T);
            const window_raw<T> wr = issue_window<T, true>(brow, bstate, t0, a.L, a.W);
            const typename io8<T>::raw rg = io8<T>::load_buf(bgrow, t0 < a.L ? (uint32_t)t0 * esz : BUF_OFF);
            const typename io4<T>::raw rgn = io4<T>::load_buf(bgrow, t0 + 8 < a.L ? (uint32_t)(t0 + 8) * esz : BUF_OFF);
            unpack_window<T, true>(wr, t0, xs, xn);
            io8<T>::unpack(rg, g);
            io4<T>::unpack(rgn, gn);
        } else {
            load_window<T, VEC>(row, state_row, t0, a.L, a.W, xs);
            io8<T>::unpack(io8<T>::template load<VEC>(grow + t0, nvalid), g);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (SILU) {
                const float v = conv_at(k4, bias, xs + j);
                const float s = sigmoid_fast(v);
                dv[j] = g[j] * s * fmaf(v, 1.0f - s, 1.0f);
            } else {
                dv[j] = g[j];
            }
        }
        // dv of the three steps after the slice: the next lane's first three, except for
        // the last lane of the wave, which works them out from global memory.
#pragma unroll
        for (int j = 0; j < HALO; ++j) {
            const float nb = __shfl_down(dv[j], 1);
            dv[8 + j] = (lane < WAVE - 1 && t0 + 8 + j < a.L) ? nb : 0.0f;
        }
        if (lane == WAVE - 1 && t0 + 8 < a.L) {
            float xe[2 * HALO];   // x[t0+5 .. t0+10]
#pragma unroll
            for (int j = 0; j < 2 * HALO; ++j) {
                if constexpr (VEC) xe[j] = j < HALO ? xs[HALO + 5 + j] : xn[j - HALO];
                else xe[j] = (t0 + 5 + j < a.L) ? io_to_f32<T>(row[t0 + 5 + j]) : 0.0f;
            }
#pragma unroll
            for (int j = 0; j < HALO; ++j) {
                float gj;
                if constexpr (VEC) gj = gn[j];
                else gj = (t0 + 8 + j < a.L) ? io_to_f32<T>(grow[t0 + 8 + j]) : 0.0f;
                if (SILU) {
                    const float v = conv_at(k4, bias, xe + j);
                    const float s = sigmoid_fast(v);
                    dv[8 + j] = gj * s * fmaf(v, 1.0f - s, 1.0f);
                } else {
                    dv[8 + j] = gj;
                }
            }
        }
        float o[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            o[j] = fmaf(k4[0], dv[j + 3], fmaf(k4[1], dv[j + 2], fmaf(k4[2], dv[j + 1], k4[3] * dv[j])));
            gb += dv[j];
#pragma unroll
            for (int i = 0; i < TAPS; ++i) gk[i] = fmaf(dv[j], xs[j + i], gk[i]);
        }
        io8<T>::template store<VEC>(static_cast<T*>(a.dx) + r * a.L + t0, o, nvalid);
    }

#pragma unroll
    for (int m = WAVE / 2; m >= 1; m >>= 1) {
        gb += __shfl_xor(gb, m);
#pragma unroll
        for (int i = 0; i < TAPS; ++i) gk[i] += __shfl_xor(gk[i], m);
    }
    if (lane == 0) {
#pragma unroll
        for (int i = 0; i < TAPS; ++i) {
            const int k = i - (TAPS - a.W);
            if (k >= 0) atomicAdd(a.dw + (size_t)d * a.W + k, gk[i]);
        }
        if (a.flags & SS_CONV_HAS_BIAS) atomicAdd(a.dbias + d, gb);
    }
}

__global__ void conv_zero_kernel(float* __restrict__ p, size_t n, float* __restrict__ q, size_t m)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0.0f;
    if (q && i < m) q[i] = 0.0f;
}

// ---- one token --------------------------------------------------------------------------------
template <typename T, bool SILU>
__global__ void conv_step_kernel(T* __restrict__ state, const T* __restrict__ x_t, const float* __restrict__ w,
                                 const float* __restrict__ bias, T* __restrict__ out_t, int rows, int D, int W)
{
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= rows) return;
    const int d = r % D;
    // Everything is requested up front, from clamped (valid) addresses and with no arithmetic on a
    // loaded value in between; masked afterwards.  Written with a test per load, the compiler
    // waited for each in turn, and the window was shifted through memory: seven round trips.
    const int lead = TAPS - W;             // unused leading slots of the right-aligned window
    T* s = state + (size_t)r * (W - 1);
    float kr[TAPS];
    T sr[HALO];
#pragma unroll
    for (int j = 0; j < TAPS; ++j) kr[j] = w[(size_t)d * W + max(j - lead, 0)];
    const T xt = x_t[r];
    const float braw = (bias ? bias : w)[bias ? d : 0];
    if (W > 1) {
#pragma unroll
        for (int j = 0; j < HALO; ++j) sr[j] = s[max(j - lead, 0)];
    } else {
#pragma unroll
        for (int j = 0; j < HALO; ++j) sr[j] = xt;
    }
    float k4[TAPS], win[TAPS];   // win[3] is the new sample
#pragma unroll
    for (int j = 0; j < TAPS; ++j) k4[j] = j >= lead ? kr[j] : 0.0f;
#pragma unroll
    for (int j = 0; j < HALO; ++j) win[j] = j >= lead ? io_to_f32<T>(sr[j]) : 0.0f;
    win[3] = io_to_f32<T>(xt);
    const float v = conv_at(k4, bias ? braw : 0.0f, win);
    out_t[r] = f32_to_io<T>(SILU ? v * sigmoid_fast(v) : v);
    // the window slides by one sample: slot j takes slot j + 1, the last slot the new sample
#pragma unroll
    for (int j = 0; j < HALO; ++j)
        if (j >= lead) s[j - lead] = j == HALO - 1 ? xt : sr[j + 1 < HALO ? j + 1 : j];
}

// ---- host ---------------------------------------------------------------------------------------
template <typename T, bool VEC>
hipError_t launch_conv_fwd_t(const ConvArgs& a, hipStream_t st)
{
    const long pieces = (a.L + PIECE - 1) / PIECE;
    const long units = (long)a.B * a.D * pieces;
    const dim3 grid((unsigned)((units + NWAVES - 1) / NWAVES));
    if (a.flags & SS_CONV_SILU) hipLaunchKernelGGL((conv_fwd_kernel<T, VEC, true>), grid, dim3(THREADS), 0, st, a);
    else hipLaunchKernelGGL((conv_fwd_kernel<T, VEC, false>), grid, dim3(THREADS), 0, st, a);
    return hipGetLastError();
}

template <typename T, bool VEC>
hipError_t launch_conv_bwd_t(const ConvArgs& a, hipStream_t st)
{
    const long pieces = (a.L + PIECE - 1) / PIECE;
    const long units = (long)a.B * pieces;
    // enough waves to keep every SIMD streaming, but no more splits than there are units
    long nsplit = (8192 + (long)a.D * NWAVES - 1) / ((long)a.D * NWAVES);
    const long most = (units + NWAVES - 1) / NWAVES;
    nsplit = nsplit < most ? nsplit : most;
    nsplit = nsplit < 1 ? 1 : (nsplit > 65535 ? 65535 : nsplit);
    const dim3 grid((unsigned)a.D, (unsigned)nsplit);
    if (a.flags & SS_CONV_SILU) hipLaunchKernelGGL((conv_bwd_kernel<T, VEC, true>), grid, dim3(THREADS), 0, st, a);
    else hipLaunchKernelGGL((conv_bwd_kernel<T, VEC, false>), grid, dim3(THREADS), 0, st, a);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_conv_t(const ConvArgs& a, bool bwd, hipStream_t st)
{
    const bool vec = a.L % 8 == 0;
    if (bwd) return vec ? launch_conv_bwd_t<T, true>(a, st) : launch_conv_bwd_t<T, false>(a, st);
    return vec ? launch_conv_fwd_t<T, true>(a, st) : launch_conv_fwd_t<T, false>(a, st);
}

}  // namespace ss

namespace {

constexpr uint32_t kConvFlags = SS_CONV_SILU | SS_CONV_HAS_BIAS | SS_CONV_HAS_STATE | SS_CONV_WRITE_STATE;
inline bool aligned_to(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

int check_conv(const ss_conv_params* p, bool for_bwd)
{
    if (!p) return SS_ERR_NULL;
    if (p->batch < 1 || p->dim < 1 || p->seqlen < 0 || p->width < 1) return SS_ERR_SHAPE;
    if (p->width > SS_CONV_MAX_WIDTH) return SS_ERR_UNSUPPORTED;
    if (p->io_dtype != SS_F32 && p->io_dtype != SS_BF16) return SS_ERR_UNSUPPORTED;
    if (p->flags & ~kConvFlags) return SS_ERR_UNSUPPORTED;
    const size_t esz = p->io_dtype == SS_BF16 ? 2 : 4;
    const bool empty = p->seqlen == 0;
    if (!p->w) return SS_ERR_NULL;
    if ((p->flags & SS_CONV_HAS_BIAS) && !p->bias) return SS_ERR_NULL;
    if (!empty && (!p->x || (!for_bwd && !p->out))) return SS_ERR_NULL;
    const bool windowed = p->width > 1;
    if (windowed && (p->flags & SS_CONV_HAS_STATE) && !p->state_in) return SS_ERR_NULL;
    if (!for_bwd && windowed && (p->flags & SS_CONV_WRITE_STATE) && !p->state_out) return SS_ERR_NULL;
    if ((p->x && !aligned_to(p->x, 16)) || (!for_bwd && p->out && !aligned_to(p->out, 16))) return SS_ERR_ALIGN;
    if ((p->state_in && !aligned_to(p->state_in, esz)) || (p->state_out && !aligned_to(p->state_out, esz))) return SS_ERR_ALIGN;
    if (!aligned_to(p->w, 4) || (p->bias && !aligned_to(p->bias, 4))) return SS_ERR_ALIGN;
    // rows are addressed through buffer resources with 31-bit offsets
    if ((size_t)p->seqlen * sizeof(float) >= ((size_t)1 << 31)) return SS_ERR_UNSUPPORTED;
    // the forward grid is one-dimensional
    const long pieces = ((long)p->seqlen + ss::PIECE - 1) / ss::PIECE;
    if ((long)p->batch * p->dim * pieces / ss::NWAVES >= 0x7fffffffL) return SS_ERR_UNSUPPORTED;
    if ((long)p->batch * pieces >= 0x7fffffffL) return SS_ERR_UNSUPPORTED;
    return SS_OK;
}

ss::ConvArgs make_conv_args(const ss_conv_params* p)
{
    ss::ConvArgs a{};
    a.B = p->batch; a.D = p->dim; a.L = p->seqlen; a.W = p->width;
    a.flags = p->flags;
    if (p->width == 1) a.flags &= ~(unsigned)(SS_CONV_HAS_STATE | SS_CONV_WRITE_STATE);
    a.x = p->x; a.state_in = p->state_in; a.w = p->w; a.bias = p->bias;
    a.out = p->out; a.state_out = p->state_out;
    return a;
}

}  // namespace

extern "C" {

int ss_conv_fwd(const ss_conv_params* p, void* stream)
{
    const int rc = check_conv(p, false);
    if (rc != SS_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const ss::ConvArgs a = make_conv_args(p);
    hipError_t e = hipSuccess;
    if (a.L == 0) {
        if (a.flags & SS_CONV_WRITE_STATE) {
            const size_t n = (size_t)a.B * a.D * (a.W - 1);
            const void* in = (a.flags & SS_CONV_HAS_STATE) ? a.state_in : nullptr;
            const dim3 grid((unsigned)((n + 255) / 256));
            if (p->io_dtype == SS_BF16)
                hipLaunchKernelGGL(ss::conv_state_copy_kernel<ss::bf16_t>, grid, dim3(256), 0, st,
                                   static_cast<const ss::bf16_t*>(in), static_cast<ss::bf16_t*>(a.state_out), n);
            else
                hipLaunchKernelGGL(ss::conv_state_copy_kernel<float>, grid, dim3(256), 0, st,
                                   static_cast<const float*>(in), static_cast<float*>(a.state_out), n);
            e = hipGetLastError();
        }
    } else {
        e = p->io_dtype == SS_BF16 ? ss::launch_conv_t<ss::bf16_t>(a, false, st) : ss::launch_conv_t<float>(a, false, st);
    }
    return e == hipSuccess ? SS_OK : SS_ERR_LAUNCH;
}

int ss_conv_bwd(const ss_conv_bwd_params* p, void* stream)
{
    if (!p) return SS_ERR_NULL;
    const int rc = check_conv(&p->fwd, true);
    if (rc != SS_OK) return rc;
    const bool empty = p->fwd.seqlen == 0;
    if (!p->dw) return SS_ERR_NULL;
    if ((p->fwd.flags & SS_CONV_HAS_BIAS) && !p->dbias) return SS_ERR_NULL;
    if (!empty && (!p->dout || !p->dx)) return SS_ERR_NULL;
    if ((p->dout && !aligned_to(p->dout, 16)) || (p->dx && !aligned_to(p->dx, 16))) return SS_ERR_ALIGN;
    if (!aligned_to(p->dw, 4) || (p->dbias && !aligned_to(p->dbias, 4))) return SS_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    ss::ConvArgs a = make_conv_args(&p->fwd);
    a.dout = p->dout; a.dx = p->dx; a.dw = p->dw;
    a.dbias = (a.flags & SS_CONV_HAS_BIAS) ? p->dbias : nullptr;
    const size_t nw = (size_t)a.D * a.W, nb = a.dbias ? (size_t)a.D : 0;
    hipLaunchKernelGGL(ss::conv_zero_kernel, dim3((unsigned)((nw + 255) / 256)), dim3(256), 0, st, a.dw, nw, a.dbias, nb);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && !empty)
        e = p->fwd.io_dtype == SS_BF16 ? ss::launch_conv_t<ss::bf16_t>(a, true, st) : ss::launch_conv_t<float>(a, true, st);
    return e == hipSuccess ? SS_OK : SS_ERR_LAUNCH;
}

int ss_conv_step(const ss_conv_step_params* p, void* stream)
{
    if (!p) return SS_ERR_NULL;
    if (p->batch < 1 || p->dim < 1 || p->width < 1) return SS_ERR_SHAPE;
    if (p->width > SS_CONV_MAX_WIDTH) return SS_ERR_UNSUPPORTED;
    if (p->io_dtype != SS_F32 && p->io_dtype != SS_BF16) return SS_ERR_UNSUPPORTED;
    if (p->flags & ~(uint32_t)(SS_CONV_SILU | SS_CONV_HAS_BIAS)) return SS_ERR_UNSUPPORTED;
    if (!p->x_t || !p->w || !p->out_t || (p->width > 1 && !p->state)) return SS_ERR_NULL;
    if ((p->flags & SS_CONV_HAS_BIAS) && !p->bias) return SS_ERR_NULL;
    const size_t esz = p->io_dtype == SS_BF16 ? 2 : 4;
    if (!aligned_to(p->x_t, esz) || !aligned_to(p->out_t, esz) || (p->state && !aligned_to(p->state, esz)) ||
        !aligned_to(p->w, 4) || (p->bias && !aligned_to(p->bias, 4)))
        return SS_ERR_ALIGN;
    const long rows = (long)p->batch * p->dim;
    if (rows >= 0x7fffffffL) return SS_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid((unsigned)((rows + 255) / 256));
    const float* bias = (p->flags & SS_CONV_HAS_BIAS) ? p->bias : nullptr;
    const bool silu = p->flags & SS_CONV_SILU;
    if (p->io_dtype == SS_BF16) {
        auto* s = static_cast<ss::bf16_t*>(p->state);
        auto* x = static_cast<const ss::bf16_t*>(p->x_t);
        auto* o = static_cast<ss::bf16_t*>(p->out_t);
        if (silu) hipLaunchKernelGGL((ss::conv_step_kernel<ss::bf16_t, true>), grid, dim3(256), 0, st, s, x, p->w, bias, o, (int)rows, p->dim, p->width);
        else hipLaunchKernelGGL((ss::conv_step_kernel<ss::bf16_t, false>), grid, dim3(256), 0, st, s, x, p->w, bias, o, (int)rows, p->dim, p->width);
    } else {
        auto* s = static_cast<float*>(p->state);
        auto* x = static_cast<const float*>(p->x_t);
        auto* o = static_cast<float*>(p->out_t);
        if (silu) hipLaunchKernelGGL((ss::conv_step_kernel<float, true>), grid, dim3(256), 0, st, s, x, p->w, bias, o, (int)rows, p->dim, p->width);
        else hipLaunchKernelGGL((ss::conv_step_kernel<float, false>), grid, dim3(256), 0, st, s, x, p->w, bias, o, (int)rows, p->dim, p->width);
    }
    return hipGetLastError() == hipSuccess ? SS_OK : SS_ERR_LAUNCH;
}

}  // extern "C"
