// The layer's projections (Algorithm 2 with the selection functions of Section 3.2: s_B, s_C linear in
// the input; s_Delta in the low-rank form Linear_D(Linear_R(x)) of Section 3.6) and their gradients, as
// this library's own kernels.  All of them are "skinny" products: one side of each is the (D, L) matrix of a batch
// entry (u, delta, d delta, du), the other has R or R + 2N (128..160) rows, so they are bound by
// reading or writing the (B, D, L) tensor once, not by arithmetic.
//
//   gemm():  C[i] (M x N) = op(A[i]) (M x K)  op(B[i]) (K x N)  [+ C[i]],  any strides, float accumulation.
//
// gemm_generic_kernel takes every shape, stride and dtype (64 x 64 tiles through LDS, 4 x 4 outputs
// per thread on the vector ALU): the float32 layer, odd sizes and the tiny per-token products.
#include <hip/hip_runtime.h>

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

}  // namespace

int gemm(const GemmArgs& g, hipStream_t stream)
{
    if (g.M <= 0 || g.N <= 0 || g.batch <= 0) return SS_OK;
    if (g.K < 0 || !g.A || !g.B || !g.C) return SS_ERR_NULL;
    if ((g.M + GT - 1) / GT > 65535 || g.batch > 65535) return SS_ERR_UNSUPPORTED;
    if (g.bf16) return g.c_float ? launch_generic<bf16_t, float>(g, stream) : launch_generic<bf16_t, bf16_t>(g, stream);
    return launch_generic<float, float>(g, stream);
}

}  // namespace ss
