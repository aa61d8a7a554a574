// The layer's projections (Algorithm 2 with the selection functions of Section 3.2: s_B, s_C linear in
// the input; s_Delta in the low-rank form Linear_D(Linear_R(x)) of Section 3.6) and their gradients, as
// this library's own kernels.  All of them are "skinny" products: one side of each is the (D, L) matrix
// of a batch entry (u, delta, d delta, du), the other has R or R + 2N (128..160) rows, so they are
// bound by reading or writing a (B, D, L) tensor once, not by arithmetic, and are built around that:
// the big operand is read (or the big result written) exactly once, in 128-byte row pieces, and the
// small operand is shared through LDS or the L2.
//
//   gemm():  C[i] (M x N) = op(A[i]) (M x K)  op(B[i]) (K x N)  [+ C[i]],  strides in elements, float accumulation.
//
// bf16 products of the three shapes the layer needs go to v_mfma_f32_16x16x32_bf16 kernels (lane l
// supplies row, resp. column, l % 16 of an operand at the 8 contraction indices from 8 * (l / 16);
// accumulator element i is row 4 * (l / 16) + i, column l % 16):
//   gemm_nt_kernel    C = A B^T with both operands contiguous along the contraction index (the
//                     weight gradients: contraction over L).  A workgroup takes 64 rows of the big
//                     operand (a 16-row fragment per wave straight from global memory) against all
//                     <= 160 rows of the small one, staged in 64-wide slabs through LDS.
//   gemm_rows_kernel  few output rows, long contraction over the ROWS of the (K, N) operand
//                     ([r;B;C] = W_x u, dr = W_dt^T ddelta): that operand is contiguous along N, not
//                     along the contraction index, so two rows at a time are interleaved into 32-bit
//                     pairs on their way into LDS and a fragment is four such pairs.
//   gemm_cols_kernel  many output rows, short contraction (delta = W_dt r, du += W_x^T d[r;B;C]): the
//                     small (K, N) operand goes through the same pairing once per workgroup and stays
//                     in registers as fragments; the product is formed transposed so that a lane
//                     holds four consecutive columns, and leaves through an LDS tile as whole
//                     128-byte row pieces.
// gemm_generic_kernel takes every other shape, stride and dtype (64 x 64 tiles through LDS, 4 x 4
// outputs per thread on the vector ALU): the float32 layer, odd sizes and the tiny per-token products.
#include <hip/hip_runtime.h>
#include <type_traits>

#include "ss_device.h"
#include "ss_kernels.h"

namespace ss {

namespace {

template <typename T> __device__ __forceinline__ float ld(const T* p);
template <> __device__ __forceinline__ float ld<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float ld<bf16_t>(const bf16_t* p) { return bf16_to_f32(*p); }
template <typename T> __device__ __forceinline__ void st(T* p, float v);
template <> __device__ __forceinline__ void st<float>(float* p, float v) { *p = v; }
template <> __device__ __forceinline__ void st<bf16_t>(bf16_t* p, float v) { *p = bf16_t(f32_to_bf16_bits(v)); }

constexpr int GT = 64;   // tile edge
constexpr int GK = 16;   // contraction indices per step

template <typename T, typename TC>
__global__ void __launch_bounds__(256) gemm_generic_kernel(const GemmArgs g)
{
    __shared__ float As[GK][GT + 4];
    __shared__ float Bs[GK][GT + 4];
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int m0 = blockIdx.y * GT, n0 = blockIdx.x * GT;
    const long bi = blockIdx.z;
    const T* __restrict__ A = static_cast<const T*>(g.A) + bi * g.a_batch;
    const T* __restrict__ B = static_cast<const T*>(g.B) + bi * g.b_batch;
    TC* __restrict__ C = static_cast<TC*>(g.C) + bi * g.c_batch;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < g.K; k0 += GK) {
        // A tile (64 m x 16 k), B tile (16 k x 64 n): four elements each per thread, along whichever
        // index is contiguous in memory
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int idx = tid + e * 256;
            int am, ak;
            if (g.a_k == 1) { ak = idx & (GK - 1); am = idx >> 4; } else { am = idx & (GT - 1); ak = idx >> 6; }
            As[ak][am] = (m0 + am < g.M && k0 + ak < g.K) ? ld(A + (long)(m0 + am) * g.a_m + (long)(k0 + ak) * g.a_k) : 0.0f;
            int bn, bk;
            if (g.b_k == 1) { bk = idx & (GK - 1); bn = idx >> 4; } else { bn = idx & (GT - 1); bk = idx >> 6; }
            Bs[bk][bn] = (n0 + bn < g.N && k0 + bk < g.K) ? ld(B + (long)(k0 + bk) * g.b_k + (long)(n0 + bn) * g.b_n) : 0.0f;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < GK; ++k) {
            const float4 a4 = *reinterpret_cast<const float4*>(&As[k][ty * 4]);
            const float4 b4 = *reinterpret_cast<const float4*>(&Bs[k][tx * 4]);
            const float a[4] = {a4.x, a4.y, a4.z, a4.w}, b[4] = {b4.x, b4.y, b4.z, b4.w};
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty * 4 + i;
        if (m >= g.M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n >= g.N) continue;
            TC* dst = C + (long)m * g.ldc + n;
            float v = acc[i][j];
            if (g.accumulate) v += ld(dst);
            st(dst, v);
        }
    }
}

template <typename T, typename TC>
int launch_generic(const GemmArgs& g, hipStream_t stream)
{
    const dim3 grid((unsigned)((g.N + GT - 1) / GT), (unsigned)((g.M + GT - 1) / GT), (unsigned)g.batch);
    hipLaunchKernelGGL((gemm_generic_kernel<T, TC>), grid, dim3(256), 0, stream, g);
    return hipGetLastError() == hipSuccess ? SS_OK : SS_ERR_LAUNCH;
}


// ---- matrix-core kernels (bf16) -------------------------------------------------------------------
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
// 16 bytes as a native vector: copies of it are plain loads and stores (a copy of the uint4 STRUCT is a
// memcpy, and registers that are only ever memcpy'd into and out of stay in scratch memory)
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
union Frag8 { uint4 u; bf16x8_t v; };
constexpr int MAXST = 10;          // the small operand has at most 160 rows
constexpr int KSLAB = 64;          // contraction indices per step
constexpr int KP = KSLAB + 8;      // LDS pitch of a slab row (bf16): 144 bytes, 16-byte aligned, off the banks
constexpr int XPITCH = 64 + 4;     // LDS pitch of a row of pairs (32-bit)

__device__ __forceinline__ f32x4_t mfma_bf16(uint4 a, uint4 b, f32x4_t c)
{
    Frag8 fa, fb;
    fa.u = a;
    fb.u = b;
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa.v, fb.v, c, 0, 0, 0);
}

// 16-byte pieces of an (S rows) x (64 columns) slab of a row-major bf16 matrix: piece p -> row p / 8,
// columns 8 * (p % 8) ..+7; thread t takes pieces t, t + 256, ... (five cover 160 rows).  Pieces past
// row S - 1 re-read the last row and land in LDS rows that no fragment reads (the LDS slab always
// has 160 rows): a load under a per-lane condition would have to be waited for on the spot, to be
// merged with the register's old value.
__device__ __forceinline__ void slab_load(u32x4 (&x)[5], const bf16_t* __restrict__ src, long ld, int S, int k0, int tid)
{
#pragma unroll
    for (int e = 0; e < 5; ++e) {
        const int p = tid + 256 * e, row = min(p >> 3, S - 1);
        x[e] = *reinterpret_cast<const u32x4*>(src + (long)row * ld + k0 + (p & 7) * 8);
    }
}
__device__ __forceinline__ void slab_store(const u32x4 (&x)[5], bf16_t (*dst)[KP], int tid)
{
#pragma unroll
    for (int e = 0; e < 5; ++e) {
        const int p = tid + 256 * e;
        *reinterpret_cast<u32x4*>(&dst[p >> 3][(p & 7) * 8]) = x[e];
    }
}

// Two rows (contraction indices 2p and 2p + 1) of a (K, N) operand that is contiguous along N,
// eight columns each, interleaved into eight 32-bit pairs {row 2p (low half), row 2p + 1 (high half)}.
__device__ __forceinline__ void pair_rows(uint4 lo, uint4 hi, uint4& out0, uint4& out1)
{
    const uint32_t l[4] = {lo.x, lo.y, lo.z, lo.w}, h[4] = {hi.x, hi.y, hi.z, hi.w};
    uint32_t o[8];
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        o[2 * m] = (l[m] & 0xffffu) | (h[m] << 16);
        o[2 * m + 1] = (l[m] >> 16) | (h[m] & 0xffff0000u);
    }
    out0 = make_uint4(o[0], o[1], o[2], o[3]);
    out1 = make_uint4(o[4], o[5], o[6], o[7]);
}

// Both kernels below walk the contraction index in 64-wide slabs and keep PD slabs in flight: the
// requests for slab s + PD go out at the start of step s into registers (slot s % PD, named at compile
// time: the loop is unrolled PD times), step s multiplies out of LDS buffer s % 2, and slab s + 1
// moves from its registers into the other LDS buffer before the step's one barrier.  The operand that
// streams from HBM is loaded with the non-temporal hint so that it does not push the small one out
// of the L2.  Requests past the last slab re-read the last slab (never used) instead of branching, so
// that the compiler's wait counts stay those of the steady state.
constexpr int PD = 4;
constexpr long ROWS_MIN_WGS = 512;   // two workgroups of gemm_rows_kernel fit on each of the 256 CUs
constexpr int ROWS_MIN_SPLIT_K = 4096;   // shorter contractions lose more to the second launch than they gain (K = 1536: 21 -> 25 us)
__device__ __forceinline__ uint4 load16_stream(const bf16_t* p)
{
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

// C[big][small] (or, OUT_T, C[small][big]), float32, = sum_k Big[big][k] Small[small][k] per batch entry.
// grid (big rows / 64, batch).  K % (64 * PD) == 0, big rows % 64 == 0, S % 16 == 0, S <= 160.
template <bool OUT_T>
__global__ void __launch_bounds__(256) gemm_nt_kernel(const bf16_t* __restrict__ Big, long big_ld, long big_batch,
                                                       const bf16_t* __restrict__ Small, long small_ld, long small_batch,
                                                       float* __restrict__ C, long ldc, long c_batch, int S, int K)
{
    __shared__ __attribute__((aligned(16))) bf16_t Ss[2][MAXST * 16][KP];
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, g = lane >> 4, j = lane & 15;
    const int d0 = blockIdx.x * 64;
    const long b = blockIdx.y;
    const bf16_t* __restrict__ arow = Big + b * big_batch + (long)(d0 + 16 * w + j) * big_ld + 8 * g;
    const bf16_t* __restrict__ sm = Small + b * small_batch;
    const int ST = S >> 4;
    const int nsteps = K / KSLAB;
    f32x4_t acc[MAXST];
#pragma unroll
    for (int ct = 0; ct < MAXST; ++ct) acc[ct] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    // one named set of registers per slot, and the step written out per slot (a macro), so that every
    // register set is addressed statically
    u32x4 sr0[5], sr1[5], sr2[5], sr3[5];
    uint4 ar0[2], ar1[2], ar2[2], ar3[2];
#define SS_NT_ISSUE(s_, SR, AR)                                          \
    {                                                                    \
        const int k0_ = min((s_), nsteps - 1) * KSLAB;                   \
        AR[0] = load16_stream(arow + k0_);                               \
        AR[1] = load16_stream(arow + k0_ + 32);                          \
        slab_load(SR, sm, small_ld, S, k0_, tid);                        \
    }
    // step s_ out of LDS buffer BUF; this slot's registers are free again (its slab went into LDS a
    // step ago, its fragments are copied out first), the next slot's slab moves into the other buffer
#define SS_NT_STEP(s_, BUF, SR, AR, SRN)                                                                              \
    {                                                                                                                 \
        const uint4 a_cur[2] = {AR[0], AR[1]};                                                                        \
        SS_NT_ISSUE((s_) + PD, SR, AR)                                                                                \
        _Pragma("unroll") for (int ks = 0; ks < 2; ++ks)                                                              \
            _Pragma("unroll") for (int ct = 0; ct < MAXST; ++ct) if (ct < ST)                                         \
            {                                                                                                         \
                const uint4 bf = *reinterpret_cast<const uint4*>(&Ss[BUF][16 * ct + j][32 * ks + 8 * g]);             \
                acc[ct] = mfma_bf16(a_cur[ks], bf, acc[ct]);                                                          \
            }                                                                                                         \
        if ((s_) + 1 < nsteps) slab_store(SRN, Ss[(BUF) ^ 1], tid);                                                   \
        __syncthreads();                                                                                              \
    }
    SS_NT_ISSUE(0, sr0, ar0)
    __builtin_amdgcn_sched_barrier(0);
    SS_NT_ISSUE(1, sr1, ar1)
    __builtin_amdgcn_sched_barrier(0);
    SS_NT_ISSUE(2, sr2, ar2)
    __builtin_amdgcn_sched_barrier(0);
    SS_NT_ISSUE(3, sr3, ar3)
    __builtin_amdgcn_sched_barrier(0);
    slab_store(sr0, Ss[0], tid);
    __syncthreads();
    for (int s0 = 0; s0 < nsteps; s0 += PD) {
        SS_NT_STEP(s0, 0, sr0, ar0, sr1)
        SS_NT_STEP(s0 + 1, 1, sr1, ar1, sr2)
        SS_NT_STEP(s0 + 2, 0, sr2, ar2, sr3)
        SS_NT_STEP(s0 + 3, 1, sr3, ar3, sr0)
    }
#undef SS_NT_STEP
#undef SS_NT_ISSUE
    float* __restrict__ c = C + b * c_batch;
#pragma unroll
    for (int ct = 0; ct < MAXST; ++ct)
        if (ct < ST) {
            const int row = d0 + 16 * w + 4 * g, col = 16 * ct + j;
            if (OUT_T) {
                *reinterpret_cast<float4*>(c + (long)col * ldc + row) = make_float4(acc[ct][0], acc[ct][1], acc[ct][2], acc[ct][3]);
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) c[(long)(row + i) * ldc + col] = acc[ct][i];
            }
        }
}

// Out (S x N per batch entry, bf16) = W (S x K, contiguous along K) X (K x N, contiguous along N).
// grid (N / 64, batch, parts).  K % (64 * PD * parts) == 0, N % 64 == 0, S % 16 == 0, S <= 160.
// With parts > 1 workgroup (., ., z) contracts over the z-th part of K and leaves its float32 share in
// Part[z][batch entry][S][N] for rows_reduce_kernel: a product with few columns would otherwise put a single
// workgroup on a CU, with nothing to run while that one waits at its barrier.
__global__ void __launch_bounds__(256) gemm_rows_kernel(const bf16_t* __restrict__ W, long w_ld, long w_batch,
                                                         const bf16_t* __restrict__ X, long x_ld, long x_batch,
                                                         bf16_t* __restrict__ Out, long o_ld, long o_batch, int S, int K,
                                                         float* __restrict__ Part)
{
    __shared__ __attribute__((aligned(16))) bf16_t Ws[2][MAXST * 16][KP];
    __shared__ __attribute__((aligned(16))) uint32_t Xp[2][KSLAB / 2][XPITCH];
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, g = lane >> 4, j = lane & 15;
    const int n0 = blockIdx.x * 64;
    const long b = blockIdx.y;
    const int kper = K / (int)gridDim.z;
    const long kbase = (long)blockIdx.z * kper;
    const bf16_t* __restrict__ wm = W + b * w_batch + kbase;
    const int xp = tid >> 3, xo = tid & 7;   // pair of rows, group of eight columns
    const bf16_t* __restrict__ xrow = X + b * x_batch + (kbase + 2 * xp) * x_ld + n0 + 8 * xo;
    const int ST = S >> 4;
    // The four waves split the S x 64 tile two by two: wave (wv, wc) has half of the output's row tiles and
    // column tiles 2 wc, 2 wc + 1, so that every weight fragment read from LDS feeds two MFMAs (with a wave
    // per column tile each wave read the whole weight slab and LDS was the limit: 78 -> 68 us).  The same
    // split of gemm_nt_kernel doubles its global fragment loads and registers and measured slower (61 -> 88 us).
    const int wv = w >> 1, wc = w & 1;
    const int RH = (ST + 1) >> 1;
    constexpr int MAXRH = MAXST / 2;
    const int nsteps = kper / KSLAB;
    f32x4_t acc[MAXRH][2];
#pragma unroll
    for (int ri = 0; ri < MAXRH; ++ri) acc[ri][0] = acc[ri][1] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    u32x4 wr0[5], wr1[5], wr2[5], wr3[5];   // one named set of registers per slot, steps written out (see gemm_nt_kernel)
    uint4 xr0[2], xr1[2], xr2[2], xr3[2];
#define SS_ROWS_ISSUE(s_, WR, XR)                                        \
    {                                                                    \
        const long k0_ = (long)min((s_), nsteps - 1) * KSLAB;            \
        XR[0] = load16_stream(xrow + k0_ * x_ld);                        \
        XR[1] = load16_stream(xrow + (k0_ + 1) * x_ld);                  \
        slab_load(WR, wm, w_ld, S, (int)k0_, tid);                       \
    }
#define SS_ROWS_FILL(BUF, WR, XR)                                        \
    {                                                                    \
        slab_store(WR, Ws[BUF], tid);                                    \
        uint4 o0_, o1_;                                                  \
        pair_rows(XR[0], XR[1], o0_, o1_);                               \
        *reinterpret_cast<uint4*>(&Xp[BUF][xp][8 * xo]) = o0_;           \
        *reinterpret_cast<uint4*>(&Xp[BUF][xp][8 * xo + 4]) = o1_;       \
    }
#define SS_ROWS_STEP(s_, BUF, WR, XR, WRN, XRN)                                                                       \
    {                                                                                                                 \
        SS_ROWS_ISSUE((s_) + PD, WR, XR) /* this slot's slab went into LDS a step ago */                              \
        _Pragma("unroll") for (int ks = 0; ks < 2; ++ks)                                                              \
        {                                                                                                             \
            const uint32_t* xq = &Xp[BUF][16 * ks + 4 * g][32 * wc + j];                                              \
            const uint4 bf0 = make_uint4(xq[0], xq[XPITCH], xq[2 * XPITCH], xq[3 * XPITCH]);                          \
            const uint4 bf1 = make_uint4(xq[16], xq[XPITCH + 16], xq[2 * XPITCH + 16], xq[3 * XPITCH + 16]);          \
            _Pragma("unroll") for (int ri = 0; ri < MAXRH; ++ri) if (ri < RH && wv * RH + ri < ST)                    \
            {                                                                                                         \
                const uint4 af = *reinterpret_cast<const uint4*>(&Ws[BUF][16 * (wv * RH + ri) + j][32 * ks + 8 * g]); \
                acc[ri][0] = mfma_bf16(af, bf0, acc[ri][0]);                                                          \
                acc[ri][1] = mfma_bf16(af, bf1, acc[ri][1]);                                                          \
            }                                                                                                         \
        }                                                                                                             \
        if ((s_) + 1 < nsteps) SS_ROWS_FILL((BUF) ^ 1, WRN, XRN)                                                      \
        __syncthreads();                                                                                              \
    }
    SS_ROWS_ISSUE(0, wr0, xr0)
    __builtin_amdgcn_sched_barrier(0);
    SS_ROWS_ISSUE(1, wr1, xr1)
    __builtin_amdgcn_sched_barrier(0);
    SS_ROWS_ISSUE(2, wr2, xr2)
    __builtin_amdgcn_sched_barrier(0);
    SS_ROWS_ISSUE(3, wr3, xr3)
    __builtin_amdgcn_sched_barrier(0);
    SS_ROWS_FILL(0, wr0, xr0)
    __syncthreads();
    for (int s0 = 0; s0 < nsteps; s0 += PD) {
        SS_ROWS_STEP(s0, 0, wr0, xr0, wr1, xr1)
        SS_ROWS_STEP(s0 + 1, 1, wr1, xr1, wr2, xr2)
        SS_ROWS_STEP(s0 + 2, 0, wr2, xr2, wr3, xr3)
        SS_ROWS_STEP(s0 + 3, 1, wr3, xr3, wr0, xr0)
    }
#undef SS_ROWS_STEP
#undef SS_ROWS_FILL
#undef SS_ROWS_ISSUE
    if (gridDim.z > 1) {
        const long ncols = (long)gridDim.x * 64;
        float* __restrict__ pp = Part + ((long)blockIdx.z * gridDim.y + b) * S * ncols + n0 + 32 * wc + j;
#pragma unroll
        for (int ri = 0; ri < MAXRH; ++ri)
            if (ri < RH && wv * RH + ri < ST) {
#pragma unroll
                for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
                    for (int i = 0; i < 4; ++i) pp[(long)(16 * (wv * RH + ri) + 4 * g + i) * ncols + 16 * c2] = acc[ri][c2][i];
            }
        return;
    }
    bf16_t* __restrict__ o = Out + b * o_batch + n0 + 32 * wc + j;
#pragma unroll
    for (int ri = 0; ri < MAXRH; ++ri)
        if (ri < RH && wv * RH + ri < ST) {
#pragma unroll
            for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    o[(long)(16 * (wv * RH + ri) + 4 * g + i) * o_ld + 16 * c2] = bf16_t(f32_to_bf16_bits(acc[ri][c2][i]));
        }
}

// Out[b][row][8 c ..+7] (bf16) = sum over the parts of Part[part][b][row][8 c ..+7]; one thread per eight columns.
__global__ void __launch_bounds__(256) rows_reduce_kernel(const float* __restrict__ Part, int parts, long part_stride,
                                                           bf16_t* __restrict__ Out, long o_ld, long o_batch, int S, int ncols,
                                                           long items)
{
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= items) return;
    const int per_row = ncols >> 3;
    const int c8 = (int)(idx % per_row);
    const long br = idx / per_row;
    const int row = (int)(br % S);
    const long b = br / S;
    const float* __restrict__ src = Part + br * ncols + 8 * c8;
    float4 lo = *reinterpret_cast<const float4*>(src), hi = *reinterpret_cast<const float4*>(src + 4);
    for (int z = 1; z < parts; ++z) {
        const float4 l2 = *reinterpret_cast<const float4*>(src + z * part_stride);
        const float4 h2 = *reinterpret_cast<const float4*>(src + z * part_stride + 4);
        lo.x += l2.x; lo.y += l2.y; lo.z += l2.z; lo.w += l2.w;
        hi.x += h2.x; hi.y += h2.y; hi.z += h2.z; hi.w += h2.w;
    }
    uint4 o;
    o.x = f32_to_bf16_bits(lo.x) | ((uint32_t)f32_to_bf16_bits(lo.y) << 16);
    o.y = f32_to_bf16_bits(lo.z) | ((uint32_t)f32_to_bf16_bits(lo.w) << 16);
    o.z = f32_to_bf16_bits(hi.x) | ((uint32_t)f32_to_bf16_bits(hi.y) << 16);
    o.w = f32_to_bf16_bits(hi.z) | ((uint32_t)f32_to_bf16_bits(hi.w) << 16);
    *reinterpret_cast<uint4*>(Out + b * o_batch + (long)row * o_ld + 8 * c8) = o;
}

// Out (M x N per batch entry, bf16) [+]= W (M x K, contiguous along K) Y (K x N, contiguous along N).
// grid (N / 64, M / (64 * mtiles), batch), mtiles = 64-row tiles of the result per workgroup (the small operand is
// prepared once for all of them).  K % 32 == 0, K <= 160, N % 64 == 0, M % (64 * mtiles) == 0.
__global__ void __launch_bounds__(256) gemm_cols_kernel(const bf16_t* __restrict__ W, long w_ld, const bf16_t* __restrict__ Y,
                                                         long y_ld, long y_batch, bf16_t* __restrict__ Out, long o_ld, long o_batch,
                                                         int K, int accumulate, int mtiles)
{
    __shared__ __attribute__((aligned(16))) uint32_t Yp[MAXST * 8][XPITCH];        // pairs of contraction indices x 64 columns
    __shared__ __attribute__((aligned(16))) float Os[64][64 + 4];                 // a tile of the result on its way out (two of them, one barrier per tile: slower, 71 -> 76 us)
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, g = lane >> 4, j = lane & 15;
    const int n0 = blockIdx.x * 64;
    const int m_base = blockIdx.y * 64 * mtiles;
    const long b = blockIdx.z;
    const bf16_t* __restrict__ y = Y + b * y_batch + n0;
    const int KS = K >> 5;   // 32-wide contraction steps (<= 5)
    // the small operand, paired and into LDS: item p -> pair of rows p / 8, eight columns from 8 * (p % 8)
    for (int p = tid; p < (K >> 1) * 8; p += 256) {
        const int pr = p >> 3, po = p & 7;
        const uint4 lo = *reinterpret_cast<const uint4*>(y + (long)(2 * pr) * y_ld + 8 * po);
        const uint4 hi = *reinterpret_cast<const uint4*>(y + (long)(2 * pr + 1) * y_ld + 8 * po);
        uint4 o0, o1;
        pair_rows(lo, hi, o0, o1);
        *reinterpret_cast<uint4*>(&Yp[pr][8 * po]) = o0;
        *reinterpret_cast<uint4*>(&Yp[pr][8 * po + 4]) = o1;
    }
    __syncthreads();
    // ... and from there into registers as fragments: first operand of the transposed product,
    // row = column 16 ct + j of Y, contraction indices 32 ks + 8 g ..+7
    uint4 yf[4][MAXST / 2];
#pragma unroll
    for (int ct = 0; ct < 4; ++ct)
#pragma unroll
        for (int ks = 0; ks < MAXST / 2; ++ks)
            if (ks < KS) {
                const uint32_t* q = &Yp[16 * ks + 4 * g][16 * ct + j];
                yf[ct][ks] = make_uint4(q[0], q[XPITCH], q[2 * XPITCH], q[3 * XPITCH]);
            }
    const bf16_t* __restrict__ wrow = W + (long)(m_base + 16 * w + j) * w_ld + 8 * g;
    uint4 wf[MAXST / 2];
#pragma unroll
    for (int ks = 0; ks < MAXST / 2; ++ks)
        if (ks < KS) wf[ks] = *reinterpret_cast<const uint4*>(wrow + 32 * ks);
    bf16_t* __restrict__ o = Out + b * o_batch + n0;
    for (int mt = 0; mt < mtiles; ++mt) {
        const int m0 = m_base + 64 * mt;
        uint4 wc[MAXST / 2];
#pragma unroll
        for (int ks = 0; ks < MAXST / 2; ++ks) wc[ks] = wf[ks];
        if (mt + 1 < mtiles) {
#pragma unroll
            for (int ks = 0; ks < MAXST / 2; ++ks)
                if (ks < KS) wf[ks] = *reinterpret_cast<const uint4*>(wrow + (long)64 * (mt + 1) * w_ld + 32 * ks);
        }
        // earlier values of this tile, for accumulation: requested before the arithmetic
        uint4 prev[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int idx = tid + 256 * e, row = idx >> 3, pc = idx & 7;
            prev[e] = accumulate ? *reinterpret_cast<const uint4*>(o + (long)(m0 + row) * o_ld + 8 * pc) : make_uint4(0u, 0u, 0u, 0u);
        }
        f32x4_t acc[4];
#pragma unroll
        for (int ct = 0; ct < 4; ++ct) {
            acc[ct] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < MAXST / 2; ++ks)
                if (ks < KS) acc[ct] = mfma_bf16(yf[ct][ks], wc[ks], acc[ct]);   // (Y^T W^T): row 16 ct + 4 g + i of Y^T, column 16 w + j of W^T
        }
        if (mt > 0) __syncthreads();   // the previous tile has left Os
#pragma unroll
        for (int ct = 0; ct < 4; ++ct)
            *reinterpret_cast<float4*>(&Os[16 * w + j][16 * ct + 4 * g]) = make_float4(acc[ct][0], acc[ct][1], acc[ct][2], acc[ct][3]);
        __syncthreads();
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int idx = tid + 256 * e, row = idx >> 3, pc = idx & 7;
            const float4 lo = *reinterpret_cast<const float4*>(&Os[row][8 * pc]);
            const float4 hi = *reinterpret_cast<const float4*>(&Os[row][8 * pc + 4]);
            float r[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
            const uint32_t c[4] = {prev[e].x, prev[e].y, prev[e].z, prev[e].w};   // zeros unless accumulating
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                r[2 * m] += bf16_lo(c[m]);
                r[2 * m + 1] += bf16_hi(c[m]);
            }
            const uint4 v = make_uint4(pack_bf16x2(r[0], r[1]), pack_bf16x2(r[2], r[3]), pack_bf16x2(r[4], r[5]), pack_bf16x2(r[6], r[7]));
            *reinterpret_cast<uint4*>(o + (long)(m0 + row) * o_ld + 8 * pc) = v;
        }
    }
}

inline bool al16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// The matrix-core kernel for this product, if there is one; SS_ERR_UNSUPPORTED otherwise (nothing enqueued).
int launch_fast(const GemmArgs& g, hipStream_t stream)
{
    if (!g.bf16 || g.K <= 0 || !al16(g.A) || !al16(g.B) || !al16(g.C)) return SS_ERR_UNSUPPORTED;
    const bf16_t* A = static_cast<const bf16_t*>(g.A);
    const bf16_t* B = static_cast<const bf16_t*>(g.B);
    auto mult8 = [](long x) { return x % 8 == 0; };
    if (g.a_k == 1 && g.b_k == 1 && g.c_float && !g.accumulate && g.K % (KSLAB * PD) == 0 && mult8(g.a_m) && mult8(g.b_n) &&
        mult8(g.a_batch) && mult8(g.b_batch) && g.ldc % 4 == 0 && g.c_batch % 4 == 0) {
        // C = A B^T: the operand with many rows is split over workgroups and waves
        float* C = static_cast<float*>(g.C);
        if (g.N % 16 == 0 && g.N <= MAXST * 16 && g.M % 64 == 0 && g.M / 64 <= 65535) {
            hipLaunchKernelGGL(gemm_nt_kernel<false>, dim3((unsigned)(g.M / 64), (unsigned)g.batch), dim3(256), 0, stream, A, g.a_m,
                               g.a_batch, B, g.b_n, g.b_batch, C, g.ldc, g.c_batch, g.N, g.K);
            return hipGetLastError() == hipSuccess ? SS_OK : SS_ERR_LAUNCH;
        }
        if (g.M % 16 == 0 && g.M <= MAXST * 16 && g.N % 64 == 0 && g.N / 64 <= 65535) {
            hipLaunchKernelGGL(gemm_nt_kernel<true>, dim3((unsigned)(g.N / 64), (unsigned)g.batch), dim3(256), 0, stream, B, g.b_n,
                               g.b_batch, A, g.a_m, g.a_batch, C, g.ldc, g.c_batch, g.M, g.K);
            return hipGetLastError() == hipSuccess ? SS_OK : SS_ERR_LAUNCH;
        }
        return SS_ERR_UNSUPPORTED;
    }
    if (g.a_k == 1 && g.b_n == 1 && !g.c_float && g.N % 64 == 0 && g.N / 64 <= 65535 && mult8(g.a_m) && mult8(g.b_k) &&
        mult8(g.a_batch) && mult8(g.b_batch) && mult8(g.ldc) && mult8(g.c_batch)) {
        bf16_t* C = static_cast<bf16_t*>(g.C);
        if (!g.accumulate && g.M % 16 == 0 && g.M <= MAXST * 16 && g.K % (KSLAB * PD) == 0) {
            // fewer than two workgroups per CU: two parts if the workspace holds two float32 shares (headline shape: 66 -> 57 us both launches together; four parts measured slower)
            const long wgs = (long)(g.N / 64) * g.batch;
            const size_t share = (size_t)g.batch * g.M * g.N * sizeof(float);
            const int parts = (wgs < ROWS_MIN_WGS && g.K >= ROWS_MIN_SPLIT_K && g.K % (KSLAB * PD * 2) == 0 && g.split_ws && 2 * share <= g.split_ws_bytes) ? 2 : 1;
            hipLaunchKernelGGL(gemm_rows_kernel, dim3((unsigned)(g.N / 64), (unsigned)g.batch, (unsigned)parts), dim3(256), 0, stream,
                               A, g.a_m, g.a_batch, B, g.b_k, g.b_batch, C, g.ldc, g.c_batch, g.M, g.K, static_cast<float*>(g.split_ws));
            if (parts > 1) {
                const long items = (long)g.batch * g.M * (g.N / 8);
                hipLaunchKernelGGL(rows_reduce_kernel, dim3((unsigned)((items + 255) / 256)), dim3(256), 0, stream,
                                   static_cast<const float*>(g.split_ws), parts, (long)g.batch * g.M * g.N, C, g.ldc, g.c_batch, g.M,
                                   g.N, items);
            }
            return hipGetLastError() == hipSuccess ? SS_OK : SS_ERR_LAUNCH;
        }
        if (g.K % 32 == 0 && g.K <= MAXST * 16 && g.M % 64 == 0 && g.a_batch == 0) {
            // as many 64-row tiles per workgroup as divide M, up to 16, while the launch keeps >= 1024 workgroups
            int mtiles = 1;
            const long cols = (long)(g.N / 64) * g.batch;
            for (int c = 16; c > 1; c >>= 1)
                if ((g.M / 64) % c == 0 && cols * (g.M / 64 / c) >= 1024) { mtiles = c; break; }
            if (g.M / (64 * mtiles) <= 65535) {
                hipLaunchKernelGGL(gemm_cols_kernel, dim3((unsigned)(g.N / 64), (unsigned)(g.M / (64 * mtiles)), (unsigned)g.batch),
                                   dim3(256), 0, stream, A, g.a_m, B, g.b_k, g.b_batch, C, g.ldc, g.c_batch, g.K, g.accumulate ? 1 : 0, mtiles);
                return hipGetLastError() == hipSuccess ? SS_OK : SS_ERR_LAUNCH;
            }
        }
    }
    return SS_ERR_UNSUPPORTED;
}

}  // namespace

int gemm(const GemmArgs& g, hipStream_t stream)
{
    if (g.M <= 0 || g.N <= 0 || g.batch <= 0) return SS_OK;
    if (g.K < 0 || !g.C || (g.K > 0 && (!g.A || !g.B))) return SS_ERR_NULL;   // K = 0: an empty sum, operands not read
    if ((g.M + GT - 1) / GT > 65535 || g.batch > 65535) return SS_ERR_UNSUPPORTED;
    if (!g.general) {
        const int rc = launch_fast(g, stream);
        if (rc != SS_ERR_UNSUPPORTED) return rc;
    }
    if (g.bf16) return g.c_float ? launch_generic<bf16_t, float>(g, stream) : launch_generic<bf16_t, bf16_t>(g, stream);
    return launch_generic<float, float>(g, stream);
}

}  // namespace ss
