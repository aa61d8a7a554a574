// Backward selective scan with state recomputation (Appendix D, "Memory").
//
// The paper states only that the (B,L,D,N) states are recomputed in the backward pass
// rather than stored; the gradient itself is the chain rule applied to Eq. 2a/2b/4.
// With dy_t the gradient reaching y_t (after the gate), g_{t,n} the gradient reaching
// h_{t,n}, and everything per (b,d):
//     g_t,n  = C_t,n dy_t + abar_{t+1,n} g_{t+1,n}            (g_L = 0; + dh_last at t = L-1)
//     dC_t,n = sum_d dy_t h_t,n              dB_t,n = sum_d g_t,n dt_t u_t
//     dA_n   = sum_{b,t} g_t,n abar_t,n h_{t-1,n} dt_t
//     ddt_t  = sum_n g_t,n (abar_t,n h_{t-1,n} A_n + B_t,n u_t)
//     du_t   = dt_t sum_n g_t,n B_t,n + Dskip dy_t        dh0_n = abar_0,n g_0,n
// and the softplus / SiLU factors of the pointwise stages.
#include "ss_kernels.h"
#include "ss_device.h"

namespace ss {

constexpr int RED_PITCH = WAVE + 4;  // pitch (floats) of the per-wave cross-row reduction tile
constexpr int RED_VALUES = GROUP_T * STATES_PER_LANE;  // 16 values per lane and group

struct BwdSmem {
    float dt[ROWS][TPAD];   // step size
    float du[ROWS][TPAD];   // dt * u
    float dy[ROWS][TPAD];   // gradient reaching y (after the gate)
    float y[ROWS][TPAD];    // y before the gate: Dskip*u + sum over waves (only with z)
    float dd[ROWS][TPAD];   // sum_n g abar h_prev A*log2(e)
    float sb[ROWS][TPAD];   // sum_n g B
    float red[NWAVES][RED_VALUES][RED_PITCH];  // cross-row reduction tile, private to a wave
    float dbc[NWAVES][2][STATES_PER_LANE][CHUNK_T];  // this chunk's dB (0) / dC (1), private to a wave
};

// LDS traffic between lanes of ONE wave needs no barrier: a wave's LDS instructions
// execute in order.  This only stops the compiler from moving accesses across the point.
__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ void lds_add(float* p, float v)
{
    __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// Sum each of this lane's RED_VALUES values (index = step j * 4 + state k) over the 64
// lanes (rows) of the wave and add the totals to acc[k][j] (pitch CHUNK_T).  Lane l =
// (quarter p = l/16, value v = l%16) adds up 16 rows of value v; the four quarters meet in
// the LDS accumulator.
__device__ __forceinline__ void reduce_over_rows(const float (&v)[RED_VALUES], float (*red)[RED_PITCH],
                                                 float* acc, int lane)
{
#pragma unroll
    for (int i = 0; i < RED_VALUES; ++i) red[i][lane] = v[i];
    wave_lds_fence();
    const int p = lane >> 4, vi = lane & 15;
    const float4* src = reinterpret_cast<const float4*>(&red[vi][16 * p]);
    const float4 a0 = src[0], a1 = src[1], a2 = src[2], a3 = src[3];
    const float s = ((a0.x + a0.y) + (a0.z + a0.w)) + ((a1.x + a1.y) + (a1.z + a1.w)) +
                    ((a2.x + a2.y) + (a2.z + a2.w)) + ((a3.x + a3.y) + (a3.z + a3.w));
    lds_add(acc + (vi & 3) * CHUNK_T + (vi >> 2), s);
    wave_lds_fence();
}

// Same decomposition as the forward kernel (64 rows x 4 waves; wave w owns states
// 4w..4w+3 of every row), walking the chunks from last to first.  Per chunk:
//   A. (pointwise view) load u, delta, z, dout; form dt, dt*u, dy and park them in LDS;
//   B1.(state view) recompute the chunk's states from the forward pass's checkpoint,
//      keeping all 32 x 4 of them in registers; accumulate y (for dz) and dC;
//   B2.(state view) run the adjoint recurrence backwards through the chunk, carrying
//      abar*g into the next (earlier) chunk in registers; accumulate dA, dB and the two
//      per-(b,d,t) sums over n that ddelta and du need;
//   C. (pointwise view) finish du, ddelta, dz and store them.
template <typename T, bool VEC, bool FULLN>
__global__ void __launch_bounds__(THREADS, 2) scan_bwd_kernel(const BwdArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    BwdSmem& sm = *reinterpret_cast<BwdSmem*>(smem_raw);

    const FwdArgs& f = a.f;
    const int tid = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & (WAVE - 1);
    const int groups = (f.D + ROWS - 1) / ROWS;
    const int b = blockIdx.x / groups;
    const int d0 = (blockIdx.x % groups) * ROWS;
    const int L = f.L, N = f.N;
    const bool has_z = f.flags & F_HAS_Z, has_D = f.flags & F_HAS_D;
    const bool softplus = f.flags & F_DELTA_SOFTPLUS;

    // ---- pointwise view ------------------------------------------------------------------
    const int pr = tid >> 2, pq = tid & 3;
    const bool p_ok = d0 + pr < f.D;
    const int pd = p_ok ? d0 + pr : f.D - 1;
    const long prow = (long)b * f.D + pd;
    const T* __restrict__ gu = static_cast<const T*>(f.u) + prow * L;
    const T* __restrict__ gdl = static_cast<const T*>(f.delta) + prow * L;
    const T* __restrict__ gz = static_cast<const T*>(f.z) + prow * L;
    const T* __restrict__ gdo = static_cast<const T*>(a.dout) + prow * L;
    T* __restrict__ gdu = static_cast<T*>(a.du) + prow * L;
    T* __restrict__ gdd = static_cast<T*>(a.ddelta) + prow * L;
    T* __restrict__ gdz = static_cast<T*>(a.dz) + prow * L;
    const float bias = (f.flags & F_HAS_DELTA_BIAS) ? f.bias[pd] : 0.0f;
    const float Dsk = has_D ? f.Dskip[pd] : 0.0f;
    float dD_acc = 0.0f, db_acc = 0.0f;

    // ---- state view ------------------------------------------------------------------------
    const bool s_ok = d0 + lane < f.D;
    const int sd = s_ok ? d0 + lane : f.D - 1;
    const long srow = (long)b * f.D + sd;
    float A2[STATES_PER_LANE], ag[STATES_PER_LANE], dA[STATES_PER_LANE];
    const T* __restrict__ gB[STATES_PER_LANE];
    const T* __restrict__ gC[STATES_PER_LANE];
    bool n_ok[STATES_PER_LANE];
#pragma unroll
    for (int k = 0; k < STATES_PER_LANE; ++k) {
        const int n = w * STATES_PER_LANE + k;
        n_ok[k] = n < N;
        const int nc = n_ok[k] ? n : 0;
        A2[k] = n_ok[k] ? f.A[(long)sd * N + nc] * LOG2E : 0.0f;
        ag[k] = (n_ok[k] && a.dh_last) ? a.dh_last[srow * N + nc] : 0.0f;  // abar_L g_L := dh_last
        dA[k] = 0.0f;
        gB[k] = static_cast<const T*>(f.Bm) + ((long)b * N + nc) * L;
        gC[k] = static_cast<const T*>(f.Cm) + ((long)b * N + nc) * L;
    }
    float* const dbc = &sm.dbc[w][0][0][0];
    float (*const red)[RED_PITCH] = sm.red[w];

    const int nchunks = (L + CHUNK_T - 1) / CHUNK_T;
    typename io8<T>::raw ru, rd, rz, ro;
    auto issue_loads = [&](int c) {
        const int t0 = c * CHUNK_T + pq * SLICE;
        const int nv = p_ok ? min(max(L - t0, 0), SLICE) : 0;  // rows past D contribute nothing
        ru = io8<T>::template load<VEC>(gu + t0, nv);
        rd = io8<T>::template load<VEC>(gdl + t0, nv);
        ro = io8<T>::template load<VEC>(gdo + t0, nv);
        if (has_z) rz = io8<T>::template load<VEC>(gz + t0, nv);
    };
    issue_loads(nchunks - 1);

    for (int c = nchunks - 1; c >= 0; --c) {
        const int tc = c * CHUNK_T;
        const int t0 = tc + pq * SLICE;
        const int nv = p_ok ? min(max(L - t0, 0), SLICE) : 0;
        // the state entering this chunk, left by the forward pass
        const float4 hck4 = *(reinterpret_cast<const float4*>(f.ckpt + (((long)c * f.B + b) * f.D + sd) * NPAD) + w);

        // ---- A: pointwise pre-processing ---------------------------------------------------
        float u8[SLICE], sg8[SLICE], zf8[SLICE];  // u, d softplus, dout * d(gate)/dz
        {
            float v8[SLICE], z8[SLICE], o8[SLICE];
            io8<T>::unpack(ru, u8);
            io8<T>::unpack(rd, v8);
            io8<T>::unpack(ro, o8);
            if (has_z) io8<T>::unpack(rz, z8);
            float dt8[SLICE], du8[SLICE], dy8[SLICE], y8[SLICE];
#pragma unroll
            for (int j = 0; j < SLICE; ++j) {
                float x = v8[j] + bias, sp, sg;
                if (softplus) softplus_sigmoid(x, sp, sg); else { sp = x; sg = 1.0f; }
                sp = (j < nv) ? sp : 0.0f;
                dt8[j] = sp;
                sg8[j] = sg;
                du8[j] = sp * u8[j];
                float dy = o8[j];
                if (has_z) {
                    const float s = sigmoid_fast(z8[j]);
                    zf8[j] = dy * s * fmaf(z8[j], 1.0f - s, 1.0f);  // dout * d[z sigmoid(z)]/dz
                    dy *= z8[j] * s;
                }
                dy8[j] = dy;
                y8[j] = Dsk * u8[j];
            }
            auto st8 = [&](float (*tile)[TPAD], const float (&v)[SLICE]) {
                float4* p4 = reinterpret_cast<float4*>(&tile[pr][pq * SLICE]);
                p4[0] = make_float4(v[0], v[1], v[2], v[3]);
                p4[1] = make_float4(v[4], v[5], v[6], v[7]);
            };
            st8(sm.dt, dt8);
            st8(sm.du, du8);
            st8(sm.dy, dy8);
            if (has_z) st8(sm.y, y8);
            const float zero8[SLICE] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            st8(sm.dd, zero8);
            st8(sm.sb, zero8);
        }
        dbc[lane] = 0.0f; dbc[lane + 64] = 0.0f; dbc[lane + 128] = 0.0f; dbc[lane + 192] = 0.0f;
        if (c > 0) issue_loads(c - 1);  // in flight during the sweeps below
        __syncthreads();

        // ---- B1: recompute the states of the chunk -----------------------------------------
        constexpr int NG = CHUNK_T / GROUP_T;
        float hs[CHUNK_T][STATES_PER_LANE];
        const float hck[STATES_PER_LANE] = {hck4.x, hck4.y, hck4.z, hck4.w};
        {
            float h[STATES_PER_LANE] = {hck[0], hck[1], hck[2], hck[3]};
            bc_group<T> Bg[2][STATES_PER_LANE], Cg[2][STATES_PER_LANE];
            auto fetch_bc = [&](int g, int slot) {
#pragma unroll
                for (int k = 0; k < STATES_PER_LANE; ++k) {
                    Bg[slot][k] = load_bc<T, VEC, !FULLN>(gB[k], tc + g * GROUP_T, L, n_ok[k]);
                    Cg[slot][k] = load_bc<T, VEC, !FULLN>(gC[k], tc + g * GROUP_T, L, n_ok[k]);
                }
            };
            fetch_bc(0, 0);
#pragma unroll
            for (int g = 0; g < NG; ++g) {
                const int cur = g & 1;
                if (g + 1 < NG) fetch_bc(g + 1, cur ^ 1);
                const int tl = g * GROUP_T;
                const float4 dt4 = *reinterpret_cast<const float4*>(&sm.dt[lane][tl]);
                const float4 du4 = *reinterpret_cast<const float4*>(&sm.du[lane][tl]);
                const float4 dy4 = *reinterpret_cast<const float4*>(&sm.dy[lane][tl]);
                float dCv[RED_VALUES];
#pragma unroll
                for (int j = 0; j < GROUP_T; ++j) {
                    const float dt = f4_get(dt4, j), du = f4_get(du4, j), dy = f4_get(dy4, j);
                    float y = 0.0f;
#pragma unroll
                    for (int k = 0; k < STATES_PER_LANE; ++k) {
                        const float abar = exp2_fast(dt * A2[k]);
                        h[k] = fmaf(abar, h[k], du * Bg[cur][k].get(j));
                        hs[tl + j][k] = h[k];
                        if (has_z) y = fmaf(Cg[cur][k].get(j), h[k], y);
                        dCv[j * STATES_PER_LANE + k] = dy * h[k];
                    }
                    if (has_z) lds_add(&sm.y[lane][tl + j], y);
                }
                reduce_over_rows(dCv, red, dbc + STATES_PER_LANE * CHUNK_T + tl, lane);
            }
        }
        // ---- B2: adjoint recurrence, last step of the chunk first --------------------------
        {
            bc_group<T> Bg[2][STATES_PER_LANE], Cg[2][STATES_PER_LANE];
            auto fetch_bc = [&](int g, int slot) {
#pragma unroll
                for (int k = 0; k < STATES_PER_LANE; ++k) {
                    Bg[slot][k] = load_bc<T, VEC, !FULLN>(gB[k], tc + g * GROUP_T, L, n_ok[k]);
                    Cg[slot][k] = load_bc<T, VEC, !FULLN>(gC[k], tc + g * GROUP_T, L, n_ok[k]);
                }
            };
            fetch_bc(NG - 1, (NG - 1) & 1);
#pragma unroll
            for (int g = NG - 1; g >= 0; --g) {
                const int cur = g & 1;
                if (g > 0) fetch_bc(g - 1, cur ^ 1);
                const int tl = g * GROUP_T;
                const float4 dt4 = *reinterpret_cast<const float4*>(&sm.dt[lane][tl]);
                const float4 du4 = *reinterpret_cast<const float4*>(&sm.du[lane][tl]);
                const float4 dy4 = *reinterpret_cast<const float4*>(&sm.dy[lane][tl]);
                float dBv[RED_VALUES];
#pragma unroll
                for (int j = GROUP_T - 1; j >= 0; --j) {
                    const int t = tl + j;
                    const float dt = f4_get(dt4, j), du = f4_get(du4, j), dy = f4_get(dy4, j);
                    float dd = 0.0f, sb = 0.0f;
#pragma unroll
                    for (int k = 0; k < STATES_PER_LANE; ++k) {
                        const float abar = exp2_fast(dt * A2[k]);
                        const float gk = fmaf(Cg[cur][k].get(j), dy, ag[k]);   // gradient reaching h_t
                        ag[k] = abar * gk;                                      // flows on to h_{t-1}
                        const float hprev = (t > 0) ? hs[t > 0 ? t - 1 : 0][k] : hck[k];
                        const float gh = ag[k] * hprev;                         // g abar h_{t-1}
                        dA[k] = fmaf(gh, dt, dA[k]);
                        dd = fmaf(gh, A2[k], dd);
                        sb = fmaf(gk, Bg[cur][k].get(j), sb);
                        dBv[j * STATES_PER_LANE + k] = gk * du;
                    }
                    lds_add(&sm.dd[lane][t], dd);
                    lds_add(&sm.sb[lane][t], sb);
                }
                reduce_over_rows(dBv, red, dbc + tl, lane);
            }
        }
        // ---- flush this wave's dB/dC of the chunk to global memory -------------------------
        wave_lds_fence();
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int idx = i * WAVE + lane;
            const int which = idx >> 7, k = (idx >> 5) & 3, t = idx & (CHUNK_T - 1);
            const int n = w * STATES_PER_LANE + k;
            if (n < N && tc + t < L) {
                float* dst = (which ? a.dC : a.dB) + ((long)b * N + n) * L + tc + t;
                atomicAdd(dst, dbc[idx]);
            }
        }
        __syncthreads();

        // ---- C: pointwise post-processing ---------------------------------------------------
        {
            auto ld8 = [&](float (*tile)[TPAD], float (&v)[SLICE]) {
                const float4* p4 = reinterpret_cast<const float4*>(&tile[pr][pq * SLICE]);
                const float4 x = p4[0], y = p4[1];
                v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
                v[4] = y.x; v[5] = y.y; v[6] = y.z; v[7] = y.w;
            };
            float dt8[SLICE], dy8[SLICE], dd8[SLICE], sb8[SLICE], y8[SLICE];
            ld8(sm.dt, dt8);
            ld8(sm.dy, dy8);
            ld8(sm.dd, dd8);
            ld8(sm.sb, sb8);
            if (has_z) ld8(sm.y, y8);
            float du8[SLICE], dl8[SLICE], dz8[SLICE];
#pragma unroll
            for (int j = 0; j < SLICE; ++j) {
                const float ddt = fmaf(u8[j], sb8[j], LN2 * dd8[j]);
                du8[j] = fmaf(dt8[j], sb8[j], Dsk * dy8[j]);
                dl8[j] = ddt * sg8[j];
                if (has_z) dz8[j] = zf8[j] * y8[j];
                dD_acc = fmaf(dy8[j], u8[j], dD_acc);
                db_acc += (j < nv) ? dl8[j] : 0.0f;
            }
            io8<T>::template store<VEC>(gdu + t0, du8, nv);
            io8<T>::template store<VEC>(gdd + t0, dl8, nv);
            if (has_z) io8<T>::template store<VEC>(gdz + t0, dz8, nv);
        }
        // the next phase A rewrites only this thread's own tile slices before its barrier
    }

    // ---- per-row results --------------------------------------------------------------------
    if (s_ok) {
        float4* pa = reinterpret_cast<float4*>(a.dA_part + srow * NPAD) + w;
        *pa = make_float4(dA[0], dA[1], dA[2], dA[3]);
        if (a.dh0) {
#pragma unroll
            for (int k = 0; k < STATES_PER_LANE; ++k)
                if (n_ok[k]) a.dh0[srow * N + w * STATES_PER_LANE + k] = ag[k];
        }
    }
    dD_acc += __shfl_xor(dD_acc, 1);
    dD_acc += __shfl_xor(dD_acc, 2);
    db_acc += __shfl_xor(db_acc, 1);
    db_acc += __shfl_xor(db_acc, 2);
    if (p_ok && pq == 0) {
        a.dD_part[prow] = dD_acc;
        a.db_part[prow] = db_acc;
    }
}

// dB and dC are accumulated atomically by the scan kernel and must start at zero.
__global__ void zero_kernel(float* __restrict__ p0, float* __restrict__ p1, long n)
{
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) { p0[i] = 0.0f; p1[i] = 0.0f; }
}

// Sum the per-batch partials: dA (D,N), dD (D), dbias (D).  With L == 0 (no partials
// written) everything is zero.
__global__ void finalize_kernel(const BwdArgs a, int have_partials)
{
    const int d = blockIdx.x * blockDim.x / NPAD + threadIdx.x / NPAD;
    const int n = threadIdx.x % NPAD;
    if (d >= a.f.D) return;
    float sA = 0.0f, sD = 0.0f, sb = 0.0f;
    if (have_partials) {
        for (int b = 0; b < a.f.B; ++b) {
            const long row = (long)b * a.f.D + d;
            sA += a.dA_part[row * NPAD + n];
            if (n == 0) { sD += a.dD_part[row]; sb += a.db_part[row]; }
        }
    }
    if (n < a.f.N) a.dA[(long)d * a.f.N + n] = sA;
    if (n == 0) {
        if (a.dD) a.dD[d] = sD;
        if (a.dbias) a.dbias[d] = sb;
    }
}

__global__ void copy_dh_kernel(const float* __restrict__ src, float* __restrict__ dst, long n)
{
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src ? src[i] : 0.0f;
}

template <typename T, bool VEC, bool FULLN>
static int launch_scan_bwd(const BwdArgs& a, dim3 grid, hipStream_t stream)
{
    static bool configured = false;  // raising the dynamic LDS limit is needed once per kernel
    auto kern = scan_bwd_kernel<T, VEC, FULLN>;
    if (!configured) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)sizeof(BwdSmem)) != hipSuccess)
            return -1;
        configured = true;
    }
    kern<<<grid, dim3(THREADS), sizeof(BwdSmem), stream>>>(a);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

int launch_bwd(const BwdArgs& a, int io_dtype, hipStream_t stream)
{
    const FwdArgs& f = a.f;
    const int fin_blocks = (f.D * NPAD + 255) / 256;
    if (f.L == 0) {
        finalize_kernel<<<dim3(fin_blocks), dim3(256), 0, stream>>>(a, 0);
        if (a.dh0) {
            const long n = (long)f.B * f.D * f.N;
            copy_dh_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream>>>(a.dh_last, a.dh0, n);
        }
        return hipGetLastError() == hipSuccess ? 0 : -1;
    }
    const long nbc = (long)f.B * f.N * f.L;
    zero_kernel<<<dim3((unsigned)((nbc + 255) / 256)), dim3(256), 0, stream>>>(a.dB, a.dC, nbc);
    const int groups = (f.D + ROWS - 1) / ROWS;
    const dim3 grid((unsigned)(f.B * groups));
    const bool fulln = f.N == NPAD;
    int rc;
    if (io_dtype == 0) {
        if (f.vec_ok && fulln) rc = launch_scan_bwd<float, true, true>(a, grid, stream);
        else if (f.vec_ok) rc = launch_scan_bwd<float, true, false>(a, grid, stream);
        else rc = launch_scan_bwd<float, false, false>(a, grid, stream);
    } else {
        if (f.vec_ok && fulln) rc = launch_scan_bwd<bf16_t, true, true>(a, grid, stream);
        else if (f.vec_ok) rc = launch_scan_bwd<bf16_t, true, false>(a, grid, stream);
        else rc = launch_scan_bwd<bf16_t, false, false>(a, grid, stream);
    }
    if (rc != 0) return rc;
    finalize_kernel<<<dim3(fin_blocks), dim3(256), 0, stream>>>(a, 1);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // namespace ss
