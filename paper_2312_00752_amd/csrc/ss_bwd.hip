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
//
// Complex state (CPLX): a lane's slots (k, k+1) are (re, im) of one complex state, the step is the
// real 2x2 map  (hr, hi) <- M (hr, hi) + dt u (Br, Bi),  M = [[abr, -abi], [abi, abr]],
// abar = abr + i abi = exp(dt (Ar + i Ai)), and y = Cr hr - Ci hi.  With (gr, gi) the gradient
// reaching (hr, hi):  (gr, gi) = (Cr, -Ci) dy + M^T (gr, gi)+,   dCr = dy hr, dCi = -dy hi,
// dBr = gr dt u, dBi = gi dt u,   and with  P = d_abr abr + d_abi abi,  Q = -d_abr abi + d_abi abr,
// d_abr = gr hr- + gi hi-,  d_abi = -gr hi- + gi hr-  (h- the previous state):
// ddt += Ar P + Ai Q + (gr Br + gi Bi) u,   dAr += dt P,   dAi += dt Q,   du += dt (gr Br + gi Bi).
#include <atomic>
#include <type_traits>

#include "ss_kernels.h"
#include "ss_device.h"

namespace ss {

constexpr int BT = CKPT_T;                // steps per backward block (one checkpoint each)
constexpr int BSL = BT * ROWS / THREADS;  // 4 steps per thread in the pointwise view
constexpr int BPAD = BT + 4;              // LDS row pitch (floats) of (row, t) tiles
constexpr int RED_PITCH = WAVE + 4;       // pitch (floats) of the per-wave cross-row reduction tile
constexpr int RED_VALUES = GROUP_T * STATES_PER_LANE;  // 16 values per lane and group

struct BwdSmem {
    float dt[ROWS][BPAD];           // step size
    float du[ROWS][BPAD];           // dt * u
    float dy[ROWS][BPAD];           // gradient reaching y (after the gate)
    float pdd[NWAVES][ROWS][BPAD];  // per wave: sum over its states of g abar h_prev A*log2(e)
    float psb[NWAVES][ROWS][BPAD];  // per wave: sum over its states of g B
    float red[NWAVES][RED_VALUES][RED_PITCH];    // cross-row reduction tile, private to a wave
    float dbc[NWAVES][2][STATES_PER_LANE][BT];   // this block's dB (0) / dC (1), private to a wave
};

// LDS traffic between lanes of ONE wave needs no barrier: a wave's LDS instructions
// execute in order.  This only stops the compiler from moving accesses across the point.
__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// x summed over lanes l, l^16, l^32, l^48 (result in every lane): two half/row swaps
__device__ __forceinline__ float sum_over_lane_quarters(float x)
{
    const auto a = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    const float y = __uint_as_float(a[0]) + __uint_as_float(a[1]);
    const auto c = __builtin_amdgcn_permlane16_swap(__float_as_uint(y), __float_as_uint(y), false, false);
    return __uint_as_float(c[0]) + __uint_as_float(c[1]);
}

// Sum over the 64 lanes (rows) of a wave of each of a lane's RED_VALUES values (index =
// step j * 4 + state k), in two halves so that the LDS round trip of one group of steps
// overlaps the arithmetic of the next: reduce_put parks the values in a [value][row] LDS
// tile; reduce_take, called one group later, has lane l = (quarter p = l/16, value v = l%16)
// add up 16 rows of value v, combines the four quarters with lane swaps and stores the
// totals to acc[k][j] (pitch BT).
__device__ __forceinline__ void reduce_put(const float (&v)[RED_VALUES], float (*red)[RED_PITCH], int lane)
{
#pragma unroll
    for (int i = 0; i < RED_VALUES; ++i) red[i][lane] = v[i];
    wave_lds_fence();
}
__device__ __forceinline__ void reduce_take(float (*red)[RED_PITCH], float* acc, int lane)
{
    const int p = lane >> 4, vi = lane & 15;
    const float4* src = reinterpret_cast<const float4*>(&red[vi][16 * p]);
    const float4 a0 = src[0], a1 = src[1], a2 = src[2], a3 = src[3];
    float s = ((a0.x + a0.y) + (a0.z + a0.w)) + ((a1.x + a1.y) + (a1.z + a1.w)) +
              ((a2.x + a2.y) + (a2.z + a2.w)) + ((a3.x + a3.y) + (a3.z + a3.w));
    s = sum_over_lane_quarters(s);
    if (p == 0) acc[(vi & 3) * BT + (vi >> 2)] = s;
    wave_lds_fence();
}
// The same for a kernel built for SPL slots per lane: a group of steps then yields 4 * SPL values, and the
// 16-value tile takes 4 / SPL groups before it is summed.  Value row = (group within the tile) * 4 SPL +
// step j * SPL + slot k; the totals of slot k at step t of the block go to acc[k * BT + t].
template <int SPL>
__device__ __forceinline__ void reduce_put_n(const float (&v)[RED_VALUES], float (*red)[RED_PITCH], int lane, int g)
{
    constexpr int GPT = STATES_PER_LANE / SPL;   // groups per tile
    const int base = (g % GPT) * GROUP_T * SPL;
#pragma unroll
    for (int j = 0; j < GROUP_T; ++j)
#pragma unroll
        for (int k = 0; k < SPL; ++k) red[base + j * SPL + k][lane] = v[j * STATES_PER_LANE + k];
    wave_lds_fence();
}
template <int SPL>
__device__ __forceinline__ void reduce_take_n(float (*red)[RED_PITCH], float* acc, int lane, int g_first)   // g_first: lowest group in the tile
{
    constexpr int GPT = STATES_PER_LANE / SPL;
    const int p = lane >> 4, vi = lane & 15;
    const float4* src = reinterpret_cast<const float4*>(&red[vi][16 * p]);
    const float4 a0 = src[0], a1 = src[1], a2 = src[2], a3 = src[3];
    float s = ((a0.x + a0.y) + (a0.z + a0.w)) + ((a1.x + a1.y) + (a1.z + a1.w)) +
              ((a2.x + a2.y) + (a2.z + a2.w)) + ((a3.x + a3.y) + (a3.z + a3.w));
    s = sum_over_lane_quarters(s);
    const int gi = vi / (GROUP_T * SPL), j = (vi % (GROUP_T * SPL)) / SPL, k = vi % SPL;
    if (p == 0) acc[k * BT + (g_first + gi) * GROUP_T + j] = s;
    wave_lds_fence();
}

// Same decomposition as the forward kernel (64 rows x 4 waves; wave w owns states
// 4w..4w+3 of every row), walking blocks of BT steps from last to first.  Per block:
//   A. (pointwise view) load u, delta, z, dout and the saved pre-gate y; form dt, dt*u, dy
//      and park them in LDS; dz is finished and stored here;
//   B1.(state view) recompute the block's states from the forward pass's checkpoint,
//      keeping states and decay factors (16 x 4 each) in registers; accumulate dC;
//   B2.(state view) run the adjoint recurrence backwards through the block, carrying
//      abar*g into the next (earlier) block in registers; accumulate dA and dB, and write
//      this wave's share of the two per-(b,d,t) sums over n that ddelta and du need;
//   C. (pointwise view) add the four waves' shares, finish du and ddelta, and store them.
// ZOH selects the exact zero-order-hold B-bar of Eq. 4.  With phi = (abar - 1)/A and
// q = g B u the formulas above become  ddt = sum_n abar (g h_prev A + q),
// dA_n += g abar h_prev dt + q dphi/dA,  du = sum_n g phi B + Dskip dy,  dB = sum_d g phi u;
// the LDS tile that otherwise carries dt*u then carries u.
// BCFIX (bit 0: B, bit 1: C): the operand is the time-invariant (D,N) parameter; it is held in
// registers like A and its gradient, a sum over batch and time, is accumulated per lane like
// dA instead of being reduced over the rows of the workgroup.
// The exact-ZOH and time-invariant-B/C variants need more registers than two workgroups per
// compute unit leave (they spilled hundreds); they are built for one workgroup per unit instead.
// (Exact ZOH with sixteen states and whole 16-byte pieces runs on scan_bwd_dpp_kernel; this kernel
// takes its other shapes.)
template <typename T, bool VEC, bool FULLN, bool ZOH, int BCFIX = 0, bool CPLX = false>
__global__ void __launch_bounds__(THREADS, (ZOH || BCFIX != 0) ? 1 : 2) scan_bwd_kernel(const BwdArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    BwdSmem& sm = *reinterpret_cast<BwdSmem*>(smem_raw);

    const FwdArgs& f = a.f;
    const int tid = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & (WAVE - 1);
    const int groups = (f.D + ROWS - 1) / ROWS;
    const unsigned bx = xcd_contiguous(blockIdx.x, gridDim.x);  // one batch entry's row groups per XCD (see scan_fwd_kernel)
    const int b = bx / groups;
    const int d0 = (bx % groups) * ROWS;
    const int L = f.L, N = f.N, NS = f.NS;
    const bool has_z = f.flags & F_HAS_Z, has_D = f.flags & F_HAS_D;
    const bool softplus = f.flags & F_DELTA_SOFTPLUS;
    const int seg = blockIdx.y;  // segment of the sequence (see scan_fwd_kernel)
    const int blk_begin = seg * (f.seg_len / BT);
    const int blk_end = min((L + BT - 1) / BT, (seg + 1) * (f.seg_len / BT));
    const long seg_rows = (long)seg * f.B * f.D;

    // ---- pointwise view: thread -> (row pr, 4-step slice pq) -----------------------------
    const int pr = pointwise_row_pitch5(tid), pq = tid & 3;   // BPAD = 20 floats
    const bool p_ok = d0 + pr < f.D;
    const int pd = p_ok ? d0 + pr : f.D - 1;
    const long prow = (long)b * f.D + pd;
    const T* __restrict__ gu = static_cast<const T*>(f.u) + prow * L;
    const T* __restrict__ gdl = static_cast<const T*>(f.delta) + prow * L;
    const T* __restrict__ gz = static_cast<const T*>(f.z) + prow * L;
    const T* __restrict__ gy = static_cast<const T*>(f.ysave) + prow * L;
    const T* __restrict__ gdo = static_cast<const T*>(a.dout) + prow * L;
    T* __restrict__ gdu = static_cast<T*>(a.du) + prow * L;
    T* __restrict__ gdd = static_cast<T*>(a.ddelta) + prow * L;
    T* __restrict__ gdz = static_cast<T*>(a.dz) + prow * L;
    const float bias = (f.flags & F_HAS_DELTA_BIAS) ? f.bias[pd] : 0.0f;
    const float Dsk = has_D ? f.Dskip[pd] : 0.0f;
    float dD_acc = 0.0f, db_acc = 0.0f;

    // ---- state view: lane -> row, wave -> states 4w..4w+3 --------------------------------
    const bool s_ok = d0 + lane < f.D;
    const int sd = s_ok ? d0 + lane : f.D - 1;
    const long srow = (long)b * f.D + sd;
    constexpr bool BFIX = BCFIX & 1, CFIX = BCFIX & 2;
    float A2[STATES_PER_LANE], An[STATES_PER_LANE], invA[STATES_PER_LANE], ag[STATES_PER_LANE], dA[STATES_PER_LANE];
    float Bf[STATES_PER_LANE], Cf[STATES_PER_LANE], dBf[STATES_PER_LANE], dCf[STATES_PER_LANE];
    const T* __restrict__ gB[STATES_PER_LANE];
    const T* __restrict__ gC[STATES_PER_LANE];
    bool n_ok[STATES_PER_LANE];
#pragma unroll
    for (int k = 0; k < STATES_PER_LANE; ++k) {
        const int n = w * STATES_PER_LANE + k;
        n_ok[k] = n < N;
        const int nc = n_ok[k] ? n : 0;
        An[k] = n_ok[k] ? f.A[(long)sd * NS + nc] : 0.0f;
        A2[k] = An[k] * LOG2E;
        invA[k] = An[k] != 0.0f ? 1.0f / An[k] : 0.0f;
        if (seg == f.nseg - 1) ag[k] = (n_ok[k] && a.dh_last) ? a.dh_last[srow * NS + nc] : 0.0f;  // abar_L g_L := dh_last
        else ag[k] = a.seg_g[(seg_rows + srow) * NPAD + w * STATES_PER_LANE + k];
        dA[k] = 0.0f;
        gB[k] = BFIX ? nullptr : static_cast<const T*>(f.Bm) + (long)b * f.bc_bstride + (long)nc * L;
        gC[k] = CFIX ? nullptr : static_cast<const T*>(f.Cm) + (long)b * f.bc_bstride + (long)nc * L;
        Bf[k] = (BFIX && n_ok[k]) ? static_cast<const float*>(f.Bm)[(long)sd * NS + nc] : 0.0f;
        Cf[k] = (CFIX && n_ok[k]) ? static_cast<const float*>(f.Cm)[(long)sd * NS + nc] : 0.0f;
        dBf[k] = 0.0f;
        dCf[k] = 0.0f;
    }
    const void* const touchB = BFIX ? f.Cm : f.Bm;   // the selective operands, if any
    const void* const touchC = CFIX ? f.Bm : f.Cm;
    float* const dbc = &sm.dbc[w][0][0][0];
    float (*const red)[RED_PITCH] = sm.red[w];

    const int nblocks = blk_end;
    // Loads are issued for 64 bytes of a row at a time (an aligned pair of bf16 blocks, one
    // float block), so that neighbouring pieces of a cache line are requested together; more
    // blocks per group would not fit the register budget.  slot = block index mod LG.
    constexpr int LG = 64 / (BT * (int)sizeof(T));
    typename io4<T>::raw ru[LG], rd[LG], rz[LG], ro[LG], ry[LG];
    auto issue_group = [&](int grp) {
#pragma unroll
        for (int s = 0; s < LG; ++s) {
            const int blk = grp * LG + s;
            const int t0 = blk * BT + pq * BSL;
            const int nv = p_ok ? min(max(L - t0, 0), BSL) : 0;  // rows past D contribute nothing
            ru[s] = io4<T>::template load<VEC>(gu + t0, nv);
            rd[s] = io4<T>::template load<VEC>(gdl + t0, nv);
            ro[s] = io4<T>::template load<VEC>(gdo + t0, nv);
            if (has_z) {
                rz[s] = io4<T>::template load<VEC>(gz + t0, nv);
                ry[s] = io4<T>::template load<VEC>(gy + t0, nv);
            }
        }
    };
    issue_group((nblocks - 1) / LG);
    uint32_t touched = 0u;
    if (BCFIX != 3) touched = touch_bc<T>(touchB, touchC, b, f.bc_bstride, N, L, w, lane, (nblocks - 1) * BT);

    auto load_ckpt = [&](int blk) {
        return *(reinterpret_cast<const float4*>(f.ckpt + (((long)blk * f.B + b) * f.D + sd) * NPAD) + w);
    };
    float4 hck_next = load_ckpt(nblocks - 1);
    for (int blk = nblocks - 1; blk >= blk_begin; --blk) {
        const int tc = blk * BT;
        consume_touch(touched);
        if (BCFIX != 3) touched = touch_bc<T>(touchB, touchC, b, f.bc_bstride, N, L, w, lane, (blk - 1) * BT);
        const int t0 = tc + pq * BSL;
        const int nv = p_ok ? min(max(L - t0, 0), BSL) : 0;
        // The state entering this block, left by the forward pass, was requested a block ago:
        // memory operations retire in order, so a wait for a load issued here would also wait
        // for every store and atomic of the previous block.
        const float4 hck4 = hck_next;
        if (blk > blk_begin) hck_next = load_ckpt(blk - 1);

        // ---- A: pointwise pre-processing ---------------------------------------------------
        float u4[BSL], sg4[BSL];  // u and d softplus(x)/dx, needed again in C
        {
            float v4[BSL], o4[BSL], dt4[BSL], du4[BSL], dy4[BSL];
            float z4[BSL], y4[BSL];
            const int slot = blk & (LG - 1);  // uniform
#pragma unroll
            for (int s = 0; s < LG; ++s) {  // unrolled so the register arrays stay statically indexed
                if (slot == s) {
                    io4<T>::unpack(ru[s], u4); io4<T>::unpack(rd[s], v4); io4<T>::unpack(ro[s], o4);
                    if (has_z) { io4<T>::unpack(rz[s], z4); io4<T>::unpack(ry[s], y4); }
                }
            }
#pragma unroll
            for (int j = 0; j < BSL; ++j) {
                float x = v4[j] + bias, sp, sg;
                if (softplus) softplus_sigmoid(x, sp, sg); else { sp = x; sg = 1.0f; }
                sp = (j < nv) ? sp : 0.0f;
                dt4[j] = sp;
                sg4[j] = sg;
                du4[j] = ZOH ? u4[j] : sp * u4[j];
                dy4[j] = o4[j];
            }
            if (has_z) {
                float dz4[BSL];
#pragma unroll
                for (int j = 0; j < BSL; ++j) {
                    const float s = sigmoid_fast(z4[j]);
                    dz4[j] = o4[j] * y4[j] * s * fmaf(z4[j], 1.0f - s, 1.0f);  // dout y d[z sigmoid(z)]/dz
                    dy4[j] = o4[j] * z4[j] * s;
                }
                if (a.dz) io4<T>::template store<VEC>(gdz + t0, dz4, nv);   // null for all but the first state group
            }
            *reinterpret_cast<float4*>(&sm.dt[pr][pq * BSL]) = make_float4(dt4[0], dt4[1], dt4[2], dt4[3]);
            *reinterpret_cast<float4*>(&sm.du[pr][pq * BSL]) = make_float4(du4[0], du4[1], du4[2], du4[3]);
            *reinterpret_cast<float4*>(&sm.dy[pr][pq * BSL]) = make_float4(dy4[0], dy4[1], dy4[2], dy4[3]);
        }
        if ((blk & (LG - 1)) == 0 && blk > blk_begin) issue_group(blk / LG - 1);  // in flight during the sweeps below
        __syncthreads();

        // ---- B1: recompute the states of the block -----------------------------------------
        // The two workgroups of a CU meet wave by wave on each SIMD.  The long state phases run at a raised
        // wave priority (the adjoint phase highest) and the short pointwise phases, which end in barriers, at the
        // default one: measured 6-8 % on this kernel and 3.7 % on the forward kernel.
        __builtin_amdgcn_s_setprio(2);
        constexpr int NG = BT / GROUP_T;
        float hs[BT][STATES_PER_LANE], as[BT][STATES_PER_LANE];
        const float hck[STATES_PER_LANE] = {hck4.x, hck4.y, hck4.z, hck4.w};
        {
            float h[STATES_PER_LANE] = {hck[0], hck[1], hck[2], hck[3]};
#pragma unroll
            for (int g = 0; g < NG; ++g) {
                bc_group<T> Bg[STATES_PER_LANE];
#pragma unroll
                for (int k = 0; k < STATES_PER_LANE; ++k)
                    if (!BFIX) Bg[k] = load_bc<T, VEC, !FULLN>(gB[k], tc + g * GROUP_T, L, n_ok[k]);
                const int tl = g * GROUP_T;
                const float4 dt4 = *reinterpret_cast<const float4*>(&sm.dt[lane][tl]);
                const float4 du4 = *reinterpret_cast<const float4*>(&sm.du[lane][tl]);
                const float4 dy4 = *reinterpret_cast<const float4*>(&sm.dy[lane][tl]);
                float dCv[RED_VALUES];
#pragma unroll
                for (int j = 0; j < GROUP_T; ++j) {
                    const float dt = f4_get(dt4, j), du = f4_get(du4, j), dy = f4_get(dy4, j);
                    if constexpr (CPLX) {
#pragma unroll
                        for (int k = 0; k < STATES_PER_LANE; k += 2) {
                            const cplx ab = complex_decay(dt, A2[k], An[k + 1]);
                            const float br = du * (BFIX ? Bf[k] : Bg[k].get(j));
                            const float bi = du * (BFIX ? Bf[k + 1] : Bg[k + 1].get(j));
                            const float hr = fmaf(ab.re, h[k], fmaf(-ab.im, h[k + 1], br));
                            const float hi = fmaf(ab.im, h[k], fmaf(ab.re, h[k + 1], bi));
                            h[k] = hr; h[k + 1] = hi;
                            as[tl + j][k] = ab.re; as[tl + j][k + 1] = ab.im;
                            hs[tl + j][k] = hr; hs[tl + j][k + 1] = hi;
                            if (CFIX) { dCf[k] = fmaf(dy, hr, dCf[k]); dCf[k + 1] = fmaf(-dy, hi, dCf[k + 1]); }
                            else { dCv[j * STATES_PER_LANE + k] = dy * hr; dCv[j * STATES_PER_LANE + k + 1] = -dy * hi; }
                        }
                    } else {
#pragma unroll
                    for (int k = 0; k < STATES_PER_LANE; ++k) {
                        const float abar = exp2_fast(dt * A2[k]);
                        float bu = du * (BFIX ? Bf[k] : Bg[k].get(j));
                        if (ZOH) bu *= zoh_phi(dt, An[k], invA[k], abar, false).phi;
                        h[k] = fmaf(abar, h[k], bu);
                        as[tl + j][k] = abar;
                        hs[tl + j][k] = h[k];
                        if (CFIX) dCf[k] = fmaf(dy, h[k], dCf[k]);
                        else dCv[j * STATES_PER_LANE + k] = dy * h[k];
                    }
                    }
                }
                if (!CFIX) {
                    if (g > 0) reduce_take(red, dbc + STATES_PER_LANE * BT + tl - GROUP_T, lane);  // previous group
                    reduce_put(dCv, red, lane);
                }
            }
            if (!CFIX) reduce_take(red, dbc + STATES_PER_LANE * BT + (NG - 1) * GROUP_T, lane);
        }
        // ---- B2: adjoint recurrence, last step of the block first --------------------------
        __builtin_amdgcn_s_setprio(3);   // the longest dependent chains of the block: above the recompute phase (another 4-6 %)
#pragma unroll
        for (int g = NG - 1; g >= 0; --g) {
            bc_group<T> Bg[STATES_PER_LANE], Cg[STATES_PER_LANE];
#pragma unroll
            for (int k = 0; k < STATES_PER_LANE; ++k) {
                if (!BFIX) Bg[k] = load_bc<T, VEC, !FULLN>(gB[k], tc + g * GROUP_T, L, n_ok[k]);
                if (!CFIX) Cg[k] = load_bc<T, VEC, !FULLN>(gC[k], tc + g * GROUP_T, L, n_ok[k]);
            }
            const int tl = g * GROUP_T;
            const float4 dt4 = *reinterpret_cast<const float4*>(&sm.dt[lane][tl]);
            const float4 du4 = *reinterpret_cast<const float4*>(&sm.du[lane][tl]);
            const float4 dy4 = *reinterpret_cast<const float4*>(&sm.dy[lane][tl]);
            float dBv[RED_VALUES], dd[GROUP_T], sb[GROUP_T];
#pragma unroll
            for (int j = GROUP_T - 1; j >= 0; --j) {
                const int t = tl + j;
                const float dt = f4_get(dt4, j), du = f4_get(du4, j), dy = f4_get(dy4, j);
                dd[j] = 0.0f;
                sb[j] = 0.0f;
                if constexpr (CPLX) {
#pragma unroll
                    for (int k = 0; k < STATES_PER_LANE; k += 2) {
                        const float Br = BFIX ? Bf[k] : Bg[k].get(j), Bi = BFIX ? Bf[k + 1] : Bg[k + 1].get(j);
                        const float gr = fmaf(CFIX ? Cf[k] : Cg[k].get(j), dy, ag[k]);
                        const float gi = fmaf(-(CFIX ? Cf[k + 1] : Cg[k + 1].get(j)), dy, ag[k + 1]);
                        const float abr = as[t][k], abi = as[t][k + 1];
                        ag[k] = fmaf(abr, gr, abi * gi);                  // M^T g flows on to h_{t-1}
                        ag[k + 1] = fmaf(abr, gi, -abi * gr);
                        const float hpr = (t > 0) ? hs[t > 0 ? t - 1 : 0][k] : hck[k];
                        const float hpi = (t > 0) ? hs[t > 0 ? t - 1 : 0][k + 1] : hck[k + 1];
                        const float d_abr = fmaf(gr, hpr, gi * hpi), d_abi = fmaf(gi, hpr, -gr * hpi);
                        const float P = fmaf(d_abr, abr, d_abi * abi), Q = fmaf(d_abi, abr, -d_abr * abi);
                        dA[k] = fmaf(P, dt, dA[k]);
                        dA[k + 1] = fmaf(Q, dt, dA[k + 1]);
                        dd[j] = fmaf(P, A2[k], fmaf(Q, A2[k + 1], dd[j]));
                        sb[j] = fmaf(gr, Br, fmaf(gi, Bi, sb[j]));
                        if (BFIX) { dBf[k] = fmaf(gr, du, dBf[k]); dBf[k + 1] = fmaf(gi, du, dBf[k + 1]); }
                        else { dBv[j * STATES_PER_LANE + k] = gr * du; dBv[j * STATES_PER_LANE + k + 1] = gi * du; }
                    }
                } else {
#pragma unroll
                for (int k = 0; k < STATES_PER_LANE; ++k) {
                    const float Bv = BFIX ? Bf[k] : Bg[k].get(j);
                    const float gk = fmaf(CFIX ? Cf[k] : Cg[k].get(j), dy, ag[k]);   // gradient reaching h_t
                    ag[k] = as[t][k] * gk;                             // flows on to h_{t-1}
                    const float hprev = (t > 0) ? hs[t > 0 ? t - 1 : 0][k] : hck[k];
                    const float gh = ag[k] * hprev;                    // g abar h_{t-1}
                    if (ZOH) {
                        const zoh_terms z = zoh_phi(dt, An[k], invA[k], as[t][k], true);
                        const float gB = gk * Bv, q = gB * du;   // du holds u here
                        dA[k] = fmaf(gh, dt, fmaf(q, z.dphi_dA, dA[k]));
                        dd[j] = fmaf(gh, An[k], fmaf(q, as[t][k], dd[j]));
                        sb[j] = fmaf(gB, z.phi, sb[j]);
                        if (BFIX) dBf[k] = fmaf(gk * z.phi, du, dBf[k]);
                        else dBv[j * STATES_PER_LANE + k] = gk * z.phi * du;
                    } else {
                        dA[k] = fmaf(gh, dt, dA[k]);
                        dd[j] = fmaf(gh, A2[k], dd[j]);
                        sb[j] = fmaf(gk, Bv, sb[j]);
                        if (BFIX) dBf[k] = fmaf(gk, du, dBf[k]);
                        else dBv[j * STATES_PER_LANE + k] = gk * du;
                    }
                }
                }
            }
            *reinterpret_cast<float4*>(&sm.pdd[w][lane][tl]) = make_float4(dd[0], dd[1], dd[2], dd[3]);
            *reinterpret_cast<float4*>(&sm.psb[w][lane][tl]) = make_float4(sb[0], sb[1], sb[2], sb[3]);
            if (!BFIX) {
                if (g < NG - 1) reduce_take(red, dbc + tl + GROUP_T, lane);  // previous (later) group
                reduce_put(dBv, red, lane);
            }
        }
        if (!BFIX) reduce_take(red, dbc, lane);
        // ---- flush this wave's dB/dC of the block to global memory -------------------------
        wave_lds_fence();
#pragma unroll
        for (int i = 0; i < 2 * STATES_PER_LANE * BT / WAVE; ++i) {
            const int idx = i * WAVE + lane;
            const int which = idx / (STATES_PER_LANE * BT), k = (idx / BT) % STATES_PER_LANE, t = idx % BT;
            const int n = w * STATES_PER_LANE + k;
            if ((which ? CFIX : BFIX)) continue;   // that gradient is not per step
            if (n < N && tc + t < L) {
                float* dst = (which ? a.dC : a.dB) + (long)b * a.dbc_bstride + (long)n * L + tc + t;
                atomicAdd(dst, dbc[idx]);
            }
        }
        __syncthreads();

        // ---- C: pointwise post-processing ---------------------------------------------------
        __builtin_amdgcn_s_setprio(0);
        {
            const float4 dt4 = *reinterpret_cast<const float4*>(&sm.dt[pr][pq * BSL]);
            const float4 dy4 = *reinterpret_cast<const float4*>(&sm.dy[pr][pq * BSL]);
            float dd4[BSL] = {0.f, 0.f, 0.f, 0.f}, sb4[BSL] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ww = 0; ww < NWAVES; ++ww) {
                const float4 x = *reinterpret_cast<const float4*>(&sm.pdd[ww][pr][pq * BSL]);
                const float4 y = *reinterpret_cast<const float4*>(&sm.psb[ww][pr][pq * BSL]);
                dd4[0] += x.x; dd4[1] += x.y; dd4[2] += x.z; dd4[3] += x.w;
                sb4[0] += y.x; sb4[1] += y.y; sb4[2] += y.z; sb4[3] += y.w;
            }
            float du4[BSL], dl4[BSL];
#pragma unroll
            for (int j = 0; j < BSL; ++j) {
                const float dt = f4_get(dt4, j), dy = f4_get(dy4, j);
                const float ddt = ZOH ? dd4[j] : fmaf(u4[j], sb4[j], LN2 * dd4[j]);
                du4[j] = ZOH ? fmaf(Dsk, dy, sb4[j]) : fmaf(dt, sb4[j], Dsk * dy);
                dl4[j] = ddt * sg4[j];
                dD_acc = fmaf(dy, u4[j], dD_acc);
                db_acc += (j < nv) ? dl4[j] : 0.0f;
            }
            if (a.acc) {  // states beyond the first 16: add to the earlier groups' du and ddelta
                float pu[BSL], pl[BSL];
                io4<T>::unpack(io4<T>::template load<VEC>(gdu + t0, nv), pu);
                io4<T>::unpack(io4<T>::template load<VEC>(gdd + t0, nv), pl);
#pragma unroll
                for (int j = 0; j < BSL; ++j) { du4[j] += pu[j]; dl4[j] += pl[j]; }
            }
            io4<T>::template store<VEC>(gdu + t0, du4, nv);
            io4<T>::template store<VEC>(gdd + t0, dl4, nv);
        }
        // the next phase A rewrites only this thread's own slices of dt/du/dy; the share
        // tiles are rewritten only after the next barrier
    }

    // ---- per-row results --------------------------------------------------------------------
    if (s_ok) {
        float4* pa = reinterpret_cast<float4*>(a.dA_part + (seg_rows + srow) * NPAD) + w;
        *pa = make_float4(dA[0], dA[1], dA[2], dA[3]);
        if (BFIX) *(reinterpret_cast<float4*>(a.dBf_part + srow * NPAD) + w) = make_float4(dBf[0], dBf[1], dBf[2], dBf[3]);
        if (CFIX) *(reinterpret_cast<float4*>(a.dCf_part + srow * NPAD) + w) = make_float4(dCf[0], dCf[1], dCf[2], dCf[3]);
        if (a.dh0 && seg == 0) {
#pragma unroll
            for (int k = 0; k < STATES_PER_LANE; ++k)
                if (n_ok[k]) a.dh0[srow * NS + w * STATES_PER_LANE + k] = ag[k];
        }
    }
    dD_acc += __shfl_xor(dD_acc, 1);
    dD_acc += __shfl_xor(dD_acc, 2);
    db_acc += __shfl_xor(db_acc, 1);
    db_acc += __shfl_xor(db_acc, 2);
    if (p_ok && pq == 0) {
        a.dD_part[seg_rows + prow] = dD_acc;
        a.db_part[seg_rows + prow] = db_acc;
    }
}

// ---- the common case: B and C as quad-broadcast operands ---------------------------------------
// Real state, first-order B-bar, selective B and C, rows of whole 16-byte pieces (L % 8 == 0): the
// same decomposition and phases as scan_bwd_kernel, but B and C do not come through the scalar
// path.  They are staged once per workgroup and block, widened to float, into a small LDS tile
// [4-step group][state][step], from which lane l of wave w reads, per group, one float4 holding
// state 4w + l % 4 at the group's four steps.  Such a register has the same four values in every
// group of four lanes, and a DPP operand with quad_perm [k,k,k,k] hands state k's value to all
// lanes at no cost: `v_mul_f32_dpp` / `v_fmac_f32_dpp` take B or C as their first operand exactly
// as the scalar-operand forms did.  What this removes: the scalar loads (which return out of order
// and share their wait counter with LDS reads, so that every LDS wait also waited for them), the
// widening of bf16 by the scalar unit, and the scalar-register spills with their v_readlane /
// v_writelane traffic on the vector ALU.  The compiler folds such a broadcast into a multiply only
// now and then and never into a multiply-add with an accumulator, so these instructions are written
// out (input_step_dpp, adjoint_step_dpp).
// All (B,D,L) tensors are addressed through per-workgroup buffer resources with ONE per-thread
// offset (they share the layout), B and C through one resource per batch entry: no 64-bit pointer
// registers, and an out-of-range offset switches a load (zeros) or a store off without a branch.
struct BwdSmemDpp {
    float dt[ROWS][BPAD];
    float du[ROWS][BPAD];
    float dy[ROWS][BPAD];
    float pdd[NWAVES][ROWS][BPAD];
    float psb[NWAVES][ROWS][BPAD];
    float red[NWAVES][RED_VALUES][RED_PITCH];
    float dbc[NWAVES][2][STATES_PER_LANE][BT];
    float bcp[2][BT / GROUP_T][NPAD][GROUP_T];   // B (0) and C (1) of the block
};


// SPL: slots per lane the state phases are built for (see scan_fwd_kernel).
// ZOH: the exact zero-order-hold B-bar of Eq. 4, b = phi B u with phi = (abar - 1)/A.  The LDS tile that
// otherwise carries dt*u then carries u, the recompute sweep keeps phi_t instead of abar_t (abar = 1 + phi A,
// one multiply-add in the adjoint sweep), and with g the gradient reaching h_t
//     ddt = sum_n abar (g h_prev A + g B u)          du = sum_n (g phi) B + Dskip dy
//     dB  = sum_d (g phi) u                          dA_n += g abar h_prev dt + g B u dphi/dA,
// where g dphi/dA = (abar g dt - g phi)/A needs neither a division nor dphi itself.  That difference cancels
// like dt A / 2 and so magnifies phi's own rounding error by 2 / |dt A|: below |dt A| = 2^-4 (and for A = 0)
// the term is g dt^2 (1/2 + x/3 + x^2/8) instead.
template <typename T, int SPL, bool ZOH = false>
__global__ void __launch_bounds__(THREADS, ZOH ? 1 : 2) scan_bwd_dpp_kernel(const BwdArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    BwdSmemDpp& sm = *reinterpret_cast<BwdSmemDpp*>(smem_raw);

    const FwdArgs& f = a.f;
    const int tid = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & (WAVE - 1);
    const int groups = (f.D + ROWS - 1) / ROWS;
    const unsigned bx = xcd_contiguous(blockIdx.x, gridDim.x);  // one batch entry's row groups per XCD (see scan_fwd_kernel)
    const int b = bx / groups;
    const int d0 = (bx % groups) * ROWS;
    const int L = f.L, N = f.N, NS = f.NS;
    const bool has_z = f.flags & F_HAS_Z, has_D = f.flags & F_HAS_D;
    const bool softplus = f.flags & F_DELTA_SOFTPLUS;
    const int seg = blockIdx.y;  // segment of the sequence (see scan_fwd_kernel)
    const int blk_begin = seg * (f.seg_len / BT);
    const int blk_end = min((L + BT - 1) / BT, (seg + 1) * (f.seg_len / BT));
    const long seg_rows = (long)seg * f.B * f.D;

    // ---- pointwise view: thread -> (row pr, 4-step slice pq) -----------------------------
    const int pr = pointwise_row_pitch5(tid), pq = tid & 3;   // BPAD = 20 floats
    const bool p_ok = d0 + pr < f.D;
    const int pd = p_ok ? d0 + pr : f.D - 1;
    const long prow = (long)b * f.D + pd;
    const float bias = (f.flags & F_HAS_DELTA_BIAS) ? f.bias[pd] : 0.0f;
    const float Dsk = has_D ? f.Dskip[pd] : 0.0f;
    float dD_acc = 0.0f, db_acc = 0.0f;
    const int rows_here = min(ROWS, f.D - d0);
    const long wg_first = ((long)b * f.D + d0) * L;
    const uint32_t wg_bytes = (uint32_t)rows_here * (uint32_t)L * (uint32_t)sizeof(T);
    const uint32_t row_off = (uint32_t)pr * (uint32_t)L * (uint32_t)sizeof(T);   // past the resource for rows past D
    auto wg_rsrc = [&](const void* base, bool on) {
        return make_rsrc(static_cast<const T*>(on ? base : f.u) + wg_first, on ? wg_bytes : 0u);
    };
    const rsrc_t bu_ = wg_rsrc(f.u, true), bd_ = wg_rsrc(f.delta, true), bo_ = wg_rsrc(a.dout, true);
    const rsrc_t bz_ = wg_rsrc(f.z, has_z), by_ = wg_rsrc(f.ysave, has_z);
    const rsrc_t bdu_ = wg_rsrc(a.du, true), bdd_ = wg_rsrc(a.ddelta, true), bdz_ = wg_rsrc(a.dz, has_z && a.dz);
    // staging view: waves 0, 1 stage B, waves 2, 3 stage C; thread -> (state s_n, pair of steps s_tp) of the block
    const int s_which = w >> 1, s_n = (tid >> 3) & (NPAD - 1), s_tp = tid & 7;
    const rsrc_t bbc_ = make_rsrc(static_cast<const T*>(s_which ? f.Cm : f.Bm) + (long)b * f.bc_bstride,
                                  (uint32_t)N * (uint32_t)L * (uint32_t)sizeof(T));
    const uint32_t bc_row_off = s_n < N ? (uint32_t)s_n * (uint32_t)L * (uint32_t)sizeof(T) : BUF_OFF;

    // ---- state view: lane -> row, wave -> states 4w..4w+3 --------------------------------
    const bool s_ok = d0 + lane < f.D;
    const int sd = s_ok ? d0 + lane : f.D - 1;
    const long srow = (long)b * f.D + sd;
    float A2[STATES_PER_LANE], dA[STATES_PER_LANE];
    float An[STATES_PER_LANE], invA[STATES_PER_LANE];   // exact ZOH only
    f32x4_t ag4;
    bool n_ok[STATES_PER_LANE];
#pragma unroll
    for (int k = 0; k < STATES_PER_LANE; ++k) {
        const int n = slot_state(w, k, f.il);
        n_ok[k] = n < N && k < SPL;
        const int nc = n_ok[k] ? n : 0;
        An[k] = n_ok[k] ? f.A[(long)sd * NS + nc] : 0.0f;
        A2[k] = An[k] * LOG2E;
        invA[k] = An[k] == 0.0f ? 0.0f : 1.0f / An[k];
        if (seg == f.nseg - 1) ag4[k] = (n_ok[k] && a.dh_last) ? a.dh_last[srow * NS + nc] : 0.0f;  // abar_L g_L := dh_last
        else ag4[k] = a.seg_g[(seg_rows + srow) * NPAD + w * STATES_PER_LANE + k];
        dA[k] = 0.0f;
    }
    float* const dbc = &sm.dbc[w][0][0][0];
    float (*const red)[RED_PITCH] = sm.red[w];
    const int pat = slot_state(w, lane & 3, f.il) * GROUP_T;   // in a group's [state][step] tile: the state of slot lane % 4

    const int nblocks = blk_end;
    // Loads are issued for 64 bytes of a row at a time (an aligned pair of bf16 blocks, one float
    // block), so that neighbouring pieces of a cache line are requested together.  slot = block index mod LG.
    constexpr int LG = 64 / (BT * (int)sizeof(T));
    typename io4<T>::raw ru[LG], rd[LG], rz[LG], ro[LG], ry[LG];
    typedef typename std::conditional<sizeof(T) == 2, uint32_t, uint2>::type bcpair_t;   // two steps of B or C
    bcpair_t rbc[LG];
    auto issue_group = [&](int grp) {
#pragma unroll
        for (int s = 0; s < LG; ++s) {
            const int blk = grp * LG + s;
            const int t0 = blk * BT + pq * BSL;
            // slices are whole or empty; rows past D lie beyond the resource
            const uint32_t off = t0 < L ? row_off + (uint32_t)t0 * (uint32_t)sizeof(T) : BUF_OFF;
            ru[s] = io4<T>::load_buf(bu_, off);
            rd[s] = io4<T>::load_buf(bd_, off);
            ro[s] = io4<T>::load_buf(bo_, off);
            rz[s] = io4<T>::load_buf(bz_, off);
            ry[s] = io4<T>::load_buf(by_, off);
            const int ts = blk * BT + 2 * s_tp;
            const uint32_t boff = ts < L ? bc_row_off + (uint32_t)ts * (uint32_t)sizeof(T) : BUF_OFF;
            if constexpr (sizeof(T) == 2) rbc[s] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(bbc_, (int)boff, 0, 0);
            else rbc[s] = buf_load8(bbc_, boff);
        }
    };
    issue_group((nblocks - 1) / LG);
    // Stores likewise: with bf16 a block is 32 bytes of a row, so the results of an odd block wait in
    // registers for the even block below it (segments start at even blocks) and the two pieces of
    // the 64-byte neighbourhood are written back to back.
    typename io4<T>::packed keep_du{}, keep_dl{}, keep_dz{};
    uint32_t keep_off = BUF_OFF;
    auto store_paired = [&](rsrc_t rs, uint32_t off, typename io4<T>::packed now, typename io4<T>::packed& keep, bool odd) {
        if constexpr (LG == 2) {
            if (odd) { keep = now; return; }
            io4<T>::store_packed(rs, keep_off, keep);   // switched off when nothing waits
        }
        io4<T>::store_packed(rs, off, now);
    };

    auto load_ckpt = [&](int blk) {
        return *(reinterpret_cast<const float4*>(f.ckpt + (((long)blk * f.B + b) * f.D + sd) * NPAD) + w);
    };
    float4 hck_next = load_ckpt(nblocks - 1);
    for (int blk = nblocks - 1; blk >= blk_begin; --blk) {
        const int tc = blk * BT;
        const int t0 = tc + pq * BSL;
        const bool live = p_ok && t0 < L;
        const uint32_t off = t0 < L ? row_off + (uint32_t)t0 * (uint32_t)sizeof(T) : BUF_OFF;
        // the state entering this block was requested a block ago (see scan_bwd_kernel)
        const float4 hck4 = hck_next;
        if (blk > blk_begin) hck_next = load_ckpt(blk - 1);

        // ---- A: pointwise pre-processing ---------------------------------------------------
        float u4[BSL], sg4[BSL];  // u and d softplus(x)/dx, needed again in C
        {
            float v4[BSL], o4[BSL], dt4[BSL], du4[BSL], dy4[BSL];
            float z4[BSL], y4[BSL];
            bcpair_t bcw{};
            const int slot = blk & (LG - 1);  // uniform
#pragma unroll
            for (int s = 0; s < LG; ++s) {  // unrolled so the register arrays stay statically indexed
                if (slot == s) {
                    io4<T>::unpack(ru[s], u4); io4<T>::unpack(rd[s], v4); io4<T>::unpack(ro[s], o4);
                    if (has_z) { io4<T>::unpack(rz[s], z4); io4<T>::unpack(ry[s], y4); }
                    bcw = rbc[s];
                }
            }
            // An empty slice reads as zeros; its steps must run with dt = 0 (the identity of the
            // recurrence) and contribute nothing: a bias of -1e30 makes softplus and its derivative
            // exactly 0 there, without a select per element.
            const float bias_eff = live ? bias : (softplus ? -1e30f : 0.0f);
            const float sg_lin = live ? 1.0f : 0.0f;
#pragma unroll
            for (int j = 0; j < BSL; ++j) {
                const float x = v4[j] + bias_eff;
                float sp, sg;
                if (softplus) softplus_sigmoid(x, sp, sg); else { sp = x; sg = sg_lin; }
                dt4[j] = sp;
                sg4[j] = sg;
                du4[j] = ZOH ? u4[j] : sp * u4[j];
                dy4[j] = o4[j];
            }
            if (has_z) {
                float dz4[BSL];
#pragma unroll
                for (int j = 0; j < BSL; ++j) {
                    const float s = sigmoid_fast(z4[j]);
                    const float zs = z4[j] * s;
                    dy4[j] = o4[j] * zs;
                    dz4[j] = (o4[j] * y4[j]) * fmaf(zs, 1.0f - s, s);   // dout y d[z sigmoid(z)]/dz
                }
                store_paired(bdz_, off, io4<T>::pack(dz4), keep_dz, blk & 1);   // switched off for all but the first state group
            }
            *reinterpret_cast<float4*>(&sm.dt[pr][pq * BSL]) = make_float4(dt4[0], dt4[1], dt4[2], dt4[3]);
            *reinterpret_cast<float4*>(&sm.du[pr][pq * BSL]) = make_float4(du4[0], du4[1], du4[2], du4[3]);
            *reinterpret_cast<float4*>(&sm.dy[pr][pq * BSL]) = make_float4(dy4[0], dy4[1], dy4[2], dy4[3]);
            float2 bc2;
            if constexpr (sizeof(T) == 2) bc2 = make_float2(bf16_lo(bcw), bf16_hi(bcw));
            else bc2 = make_float2(__uint_as_float(bcw.x), __uint_as_float(bcw.y));
            *reinterpret_cast<float2*>(&sm.bcp[s_which][s_tp >> 1][s_n][(s_tp & 1) * 2]) = bc2;
        }
        if ((blk & (LG - 1)) == 0 && blk > blk_begin) issue_group(blk / LG - 1);  // in flight during the sweeps below
        __syncthreads();

        // ---- B1: recompute the states of the block -----------------------------------------
        __builtin_amdgcn_s_setprio(2);
        constexpr int NG = BT / GROUP_T;
        constexpr int GPT = STATES_PER_LANE / SPL;   // groups of steps per tile of the cross-row reduction
        f32x4_t as4[BT], hs4[BT];   // abar_t (exact ZOH: phi_t) and h_t
        {
            f32x4_t h4 = {hck4.x, hck4.y, hck4.z, hck4.w};
#pragma unroll
            for (int g = 0; g < NG; ++g) {
                const int tl = g * GROUP_T;
                const float4 dt4 = *reinterpret_cast<const float4*>(&sm.dt[lane][tl]);
                const float4 du4 = *reinterpret_cast<const float4*>(&sm.du[lane][tl]);
                const float4 dy4 = *reinterpret_cast<const float4*>(&sm.dy[lane][tl]);
                const float4 Bp = *reinterpret_cast<const float4*>(&sm.bcp[0][g][0][0] + pat);
                float dCv[RED_VALUES];
#pragma unroll
                for (int j = 0; j < GROUP_T; ++j) {
                    const float dt = f4_get(dt4, j), du = f4_get(du4, j), dy = f4_get(dy4, j);
                    float bu[STATES_PER_LANE];
                    input_step_dpp<SPL>(bu, f4_get(Bp, j), du);
                    f32x4_t ab = {1.f, 1.f, 1.f, 1.f};
                    if constexpr (ZOH) ab = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int k = 0; k < SPL; ++k) {
                        if constexpr (ZOH) {                              // bu holds B u
                            const float x2 = dt * A2[k];
                            const float abar = exp2_fast(x2);             // Eq. 4
                            const float phi = zoh_phi_fast(dt, x2, abar, invA[k]);
                            h4[k] = fmaf(abar, h4[k], phi * bu[k]);       // Eq. 2a
                            ab[k] = phi;
                        } else {
                            ab[k] = exp2_fast(dt * A2[k]);                // Eq. 4
                            h4[k] = fmaf(ab[k], h4[k], bu[k]);            // Eq. 2a
                        }
                    }
                    as4[tl + j] = ab;
                    hs4[tl + j] = h4;
#pragma unroll
                    for (int k = 0; k < SPL; ++k) dCv[j * STATES_PER_LANE + k] = dy * h4[k];
                }
                // the tile of the previous GPT groups is summed a group later, before this group's values go in
                if (g > 0 && g % GPT == 0) reduce_take_n<SPL>(red, dbc + STATES_PER_LANE * BT, lane, g - GPT);
                reduce_put_n<SPL>(dCv, red, lane, g);
            }
            reduce_take_n<SPL>(red, dbc + STATES_PER_LANE * BT, lane, NG - GPT);
        }
        // ---- B2: adjoint recurrence, last step of the block first --------------------------
        __builtin_amdgcn_s_setprio(3);
#pragma unroll
        for (int g = NG - 1; g >= 0; --g) {
            const int tl = g * GROUP_T;
            const float4 dt4 = *reinterpret_cast<const float4*>(&sm.dt[lane][tl]);
            const float4 du4 = *reinterpret_cast<const float4*>(&sm.du[lane][tl]);
            const float4 dy4 = *reinterpret_cast<const float4*>(&sm.dy[lane][tl]);
            const float4 Bp = *reinterpret_cast<const float4*>(&sm.bcp[0][g][0][0] + pat);
            const float4 Cp = *reinterpret_cast<const float4*>(&sm.bcp[1][g][0][0] + pat);
            float dBv[RED_VALUES], dd[GROUP_T], sb[GROUP_T];
#pragma unroll
            for (int j = GROUP_T - 1; j >= 0; --j) {
                const int t = tl + j;
                const float dt = f4_get(dt4, j), du = f4_get(du4, j), dy = f4_get(dy4, j);
                dd[j] = 0.0f;
                if constexpr (ZOH) {
                    float gk[STATES_PER_LANE] = {ag4[0], ag4[1], ag4[2], ag4[3]};
                    adjoint_input_dpp<SPL>(gk, f4_get(Cp, j), dy);         // g = C dy + abar+ g+
                    float Bu[STATES_PER_LANE], gphi[STATES_PER_LANE] = {0.f, 0.f, 0.f, 0.f};
                    input_step_dpp<SPL>(Bu, f4_get(Bp, j), du);            // B u  (the tile carries u)
                    const float dt2 = dt * dt;
#pragma unroll
                    for (int k = 0; k < SPL; ++k) {
                        const float phi = as4[t][k];
                        ag4[k] = fmaf(phi, An[k], 1.0f) * gk[k];           // abar g: flows on to h_{t-1}
                        const float gh = ag4[k] * (t > 0 ? hs4[t > 0 ? t - 1 : 0][k] : f4_get(hck4, k));   // g abar h_{t-1}
                        gphi[k] = gk[k] * phi;
                        const float x2 = dt * A2[k];
                        const float direct = fmaf(ag4[k], dt, -gphi[k]) * invA[k];
                        const float series = (gk[k] * dt2) * fmaf(x2, fmaf(x2, LN2 * LN2 / 8.0f, LN2 / 3.0f), 0.5f);
                        const float gdphi = select_small(x2, ZOH_SMALL_X2_GRAD, series, direct);   // g dphi/dA
                        dA[k] = fmaf(gh, dt, fmaf(Bu[k], gdphi, dA[k]));
                        dd[j] = fmaf(gh, An[k], fmaf(Bu[k], ag4[k], dd[j]));
                        dBv[j * STATES_PER_LANE + k] = gphi[k] * du;
                    }
                    readout_step_dpp<SPL>(sb[j], f4_get(Bp, j), gphi);     // sb = sum_k B_k g_k phi_k
                } else {
                f32x4_t g4 = ag4;
                adjoint_step_dpp<SPL>(g4, sb[j], f4_get(Cp, j), f4_get(Bp, j), dy);   // g = C dy + abar+ g+;  sb = sum_k B_k g_k
#pragma unroll
                for (int k = 0; k < SPL; ++k) {
                    ag4[k] = as4[t][k] * g4[k];                         // flows on to h_{t-1}
                    const float gh = ag4[k] * (t > 0 ? hs4[t > 0 ? t - 1 : 0][k] : f4_get(hck4, k));   // g abar h_{t-1}
                    dA[k] = fmaf(gh, dt, dA[k]);
                    dd[j] = fmaf(gh, A2[k], dd[j]);
                    dBv[j * STATES_PER_LANE + k] = g4[k] * du;
                }
                }
            }
            *reinterpret_cast<float4*>(&sm.pdd[w][lane][tl]) = make_float4(dd[0], dd[1], dd[2], dd[3]);
            *reinterpret_cast<float4*>(&sm.psb[w][lane][tl]) = make_float4(sb[0], sb[1], sb[2], sb[3]);
            if (g < NG - 1 && (g + 1) % GPT == 0) reduce_take_n<SPL>(red, dbc, lane, g + 1);  // the tile of the GPT groups above
            reduce_put_n<SPL>(dBv, red, lane, g);
        }
        reduce_take_n<SPL>(red, dbc, lane, 0);
        // ---- flush this wave's dB/dC of the block to global memory -------------------------
        wave_lds_fence();
#pragma unroll
        for (int i = 0; i < 2 * STATES_PER_LANE * BT / WAVE; ++i) {
            const int idx = i * WAVE + lane;
            const int which = idx / (STATES_PER_LANE * BT), k = (idx / BT) % STATES_PER_LANE, t = idx % BT;
            const int n = slot_state(w, k, f.il);
            if (k < SPL && n < N && tc + t < L) {
                float* dst = (which ? a.dC : a.dB) + (long)b * a.dbc_bstride + (long)n * L + tc + t;
                atomicAdd(dst, dbc[idx]);
            }
        }
        __syncthreads();

        // ---- C: pointwise post-processing ---------------------------------------------------
        __builtin_amdgcn_s_setprio(0);
        {
            const float4 dt4 = *reinterpret_cast<const float4*>(&sm.dt[pr][pq * BSL]);
            const float4 dy4 = *reinterpret_cast<const float4*>(&sm.dy[pr][pq * BSL]);
            float dd4[BSL] = {0.f, 0.f, 0.f, 0.f}, sb4[BSL] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ww = 0; ww < NWAVES; ++ww) {
                const float4 x = *reinterpret_cast<const float4*>(&sm.pdd[ww][pr][pq * BSL]);
                const float4 y = *reinterpret_cast<const float4*>(&sm.psb[ww][pr][pq * BSL]);
                dd4[0] += x.x; dd4[1] += x.y; dd4[2] += x.z; dd4[3] += x.w;
                sb4[0] += y.x; sb4[1] += y.y; sb4[2] += y.z; sb4[3] += y.w;
            }
            float du4[BSL], dl4[BSL];
#pragma unroll
            for (int j = 0; j < BSL; ++j) {
                const float dt = f4_get(dt4, j), dy = f4_get(dy4, j);
                const float ddt = ZOH ? dd4[j] : fmaf(u4[j], sb4[j], LN2 * dd4[j]);
                du4[j] = ZOH ? fmaf(Dsk, dy, sb4[j]) : fmaf(dt, sb4[j], Dsk * dy);
                dl4[j] = ddt * sg4[j];             // 0 on an empty slice: its sg is 0
                dD_acc = fmaf(dy, u4[j], dD_acc);
                db_acc += dl4[j];
            }
            if (a.acc) {  // states beyond the first 16: add to the earlier groups' du and ddelta
                float pu[BSL], pl[BSL];
                io4<T>::unpack(io4<T>::load_buf(bdu_, off), pu);
                io4<T>::unpack(io4<T>::load_buf(bdd_, off), pl);
#pragma unroll
                for (int j = 0; j < BSL; ++j) { du4[j] += pu[j]; dl4[j] += pl[j]; }
            }
            store_paired(bdu_, off, io4<T>::pack(du4), keep_du, blk & 1);
            store_paired(bdd_, off, io4<T>::pack(dl4), keep_dl, blk & 1);
            if constexpr (LG == 2) keep_off = (blk & 1) ? off : BUF_OFF;
        }
    }

    // ---- per-row results --------------------------------------------------------------------
    if (s_ok) {
        float4* pa = reinterpret_cast<float4*>(a.dA_part + (seg_rows + srow) * NPAD) + w;
        *pa = make_float4(dA[0], dA[1], dA[2], dA[3]);
        if (a.dh0 && seg == 0) {
#pragma unroll
            for (int k = 0; k < STATES_PER_LANE; ++k)
                if (n_ok[k]) a.dh0[srow * NS + slot_state(w, k, f.il)] = ag4[k];
        }
    }
    dD_acc += __shfl_xor(dD_acc, 1);
    dD_acc += __shfl_xor(dD_acc, 2);
    db_acc += __shfl_xor(db_acc, 1);
    db_acc += __shfl_xor(db_acc, 2);
    if (p_ok && pq == 0) {
        a.dD_part[seg_rows + prow] = dD_acc;
        a.db_part[seg_rows + prow] = db_acc;
    }
}

// Adjoint aggregate of a segment, for a sequence split across workgroups: runs only the
// adjoint recurrence g = C dy + abar+ g+ over the segment, from a zero carry (last segment:
// from dh_last), and leaves the carry abar g at the segment's first step in seg_g.  Needs
// no states, so it is the forward kernel's loop structure walked backwards: 32-step chunks,
// dt and dy staged through LDS, C on the scalar path.
template <typename T, bool VEC, bool FULLN, bool CPLX = false, int SPL = STATES_PER_LANE>
__global__ void __launch_bounds__(THREADS) adjoint_agg_kernel(const BwdArgs a)
{
    __shared__ __attribute__((aligned(16))) float s_dt[ROWS][TPAD];
    __shared__ __attribute__((aligned(16))) float s_dy[ROWS][TPAD];
    const FwdArgs& f = a.f;
    const int tid = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & (WAVE - 1);
    const int groups = (f.D + ROWS - 1) / ROWS;
    const unsigned bx = xcd_contiguous(blockIdx.x, gridDim.x);  // one batch entry's row groups per XCD (see scan_fwd_kernel)
    const int b = bx / groups;
    const int d0 = (bx % groups) * ROWS;
    const int L = f.L, N = f.N, NS = f.NS;
    const bool has_z = f.flags & F_HAS_Z, softplus = f.flags & F_DELTA_SOFTPLUS;
    const int seg = blockIdx.y + 1;  // segment 0 passes nothing on
    const int c_begin = seg * (f.seg_len / CHUNK_T);
    const int c_end = min((L + CHUNK_T - 1) / CHUNK_T, (seg + 1) * (f.seg_len / CHUNK_T));

    const int pr = pointwise_row_pitch9(tid), pq = tid & 3;   // TPAD = 36 floats
    const bool p_ok = d0 + pr < f.D;
    const int pd = p_ok ? d0 + pr : f.D - 1;
    const long prow = (long)b * f.D + pd;
    const T* __restrict__ gdl = static_cast<const T*>(f.delta) + prow * L;
    const T* __restrict__ gz = static_cast<const T*>(f.z) + prow * L;
    const T* __restrict__ gdo = static_cast<const T*>(a.dout) + prow * L;
    const float bias = (f.flags & F_HAS_DELTA_BIAS) ? f.bias[pd] : 0.0f;

    const bool s_ok = d0 + lane < f.D;
    const int sd = s_ok ? d0 + lane : f.D - 1;
    const long srow = (long)b * f.D + sd;
    float A2[STATES_PER_LANE], An[STATES_PER_LANE], ag[STATES_PER_LANE];
    const T* __restrict__ gC[STATES_PER_LANE];
    bool n_ok[STATES_PER_LANE];
#pragma unroll
    for (int k = 0; k < STATES_PER_LANE; ++k) {
        const int n = slot_state(w, k, f.il);
        n_ok[k] = n < N && k < SPL;
        const int nc = n_ok[k] ? n : 0;
        An[k] = n_ok[k] ? f.A[(long)sd * NS + nc] : 0.0f;
        A2[k] = An[k] * LOG2E;
        ag[k] = (seg == f.nseg - 1 && n_ok[k] && a.dh_last) ? a.dh_last[srow * NS + nc] : 0.0f;
        gC[k] = static_cast<const T*>(f.Cm) + (long)b * f.bc_bstride + (long)nc * L;
    }
    typename io8<T>::raw rd, rz, ro;
    auto issue_loads = [&](int c) {
        const int t0 = c * CHUNK_T + pq * SLICE;
        const int nv = p_ok ? min(max(L - t0, 0), SLICE) : 0;
        rd = io8<T>::template load<VEC>(gdl + t0, nv);
        ro = io8<T>::template load<VEC>(gdo + t0, nv);
        if (has_z) rz = io8<T>::template load<VEC>(gz + t0, nv);
    };
    issue_loads(c_end - 1);
    uint32_t touched = touch_bc<T>(f.Cm, f.Cm, b, f.bc_bstride, N, L, w, lane, (c_end - 1) * CHUNK_T);
    for (int c = c_end - 1; c >= c_begin; --c) {
        const int tc = c * CHUNK_T;
        consume_touch(touched);
        touched = touch_bc<T>(f.Cm, f.Cm, b, f.bc_bstride, N, L, w, lane, (c - 1) * CHUNK_T);
        const int nv = p_ok ? min(max(L - (tc + pq * SLICE), 0), SLICE) : 0;
        {
            float v8[SLICE], o8[SLICE], z8[SLICE], dt8[SLICE];
            io8<T>::unpack(rd, v8);
            io8<T>::unpack(ro, o8);
            if (has_z) io8<T>::unpack(rz, z8);
#pragma unroll
            for (int j = 0; j < SLICE; ++j) {
                float x = v8[j] + bias, sp, sg;
                if (softplus) softplus_sigmoid(x, sp, sg); else sp = x;
                dt8[j] = (j < nv) ? sp : 0.0f;
                if (has_z) o8[j] *= z8[j] * sigmoid_fast(z8[j]);
            }
            float4* pd4 = reinterpret_cast<float4*>(&s_dt[pr][pq * SLICE]);
            float4* py4 = reinterpret_cast<float4*>(&s_dy[pr][pq * SLICE]);
            pd4[0] = make_float4(dt8[0], dt8[1], dt8[2], dt8[3]);
            pd4[1] = make_float4(dt8[4], dt8[5], dt8[6], dt8[7]);
            py4[0] = make_float4(o8[0], o8[1], o8[2], o8[3]);
            py4[1] = make_float4(o8[4], o8[5], o8[6], o8[7]);
        }
        if (c > c_begin) issue_loads(c - 1);
        __syncthreads();
        __builtin_amdgcn_s_setprio(2);   // as in scan_bwd_kernel: the recurrence at a raised wave priority
        constexpr int NG = CHUNK_T / GROUP_T;
#pragma unroll
        for (int g = NG - 1; g >= 0; --g) {
            bc_group<T> Cg[STATES_PER_LANE];
#pragma unroll
            for (int k = 0; k < STATES_PER_LANE; ++k)
                Cg[k] = load_bc<T, VEC, !FULLN>(gC[k], tc + g * GROUP_T, L, n_ok[k]);
            const float4 dt4 = *reinterpret_cast<const float4*>(&s_dt[lane][g * GROUP_T]);
            const float4 dy4 = *reinterpret_cast<const float4*>(&s_dy[lane][g * GROUP_T]);
#pragma unroll
            for (int j = GROUP_T - 1; j >= 0; --j) {
                const float dt = f4_get(dt4, j), dy = f4_get(dy4, j);
                if constexpr (CPLX) {
#pragma unroll
                    for (int k = 0; k < STATES_PER_LANE; k += 2) {
                        const cplx ab = complex_decay(dt, A2[k], An[k + 1]);
                        const float gr = fmaf(Cg[k].get(j), dy, ag[k]), gi = fmaf(-Cg[k + 1].get(j), dy, ag[k + 1]);
                        ag[k] = fmaf(ab.re, gr, ab.im * gi);
                        ag[k + 1] = fmaf(ab.re, gi, -ab.im * gr);
                    }
                } else {
#pragma unroll
                    for (int k = 0; k < SPL; ++k)
                        ag[k] = exp2_fast(dt * A2[k]) * fmaf(Cg[k].get(j), dy, ag[k]);
                }
            }
        }
        __builtin_amdgcn_s_setprio(0);
        __syncthreads();
    }
    if (s_ok) {
        float4* dst = reinterpret_cast<float4*>(a.seg_g + ((long)seg * f.B * f.D + srow) * NPAD) + w;
        *dst = make_float4(ag[0], ag[1], ag[2], ag[3]);
    }
}

// The adjoint aggregate on the common path (real state, selective C, L % 8 == 0): as
// adjoint_agg_kernel, with the chunk's C staged through an LDS tile and taken as a quad-broadcast
// DPP operand (see scan_bwd_dpp_kernel), buffer-addressed inputs requested two chunks ahead into
// compile-time slots, and no scalar loads.
template <typename T, int SPL>
__global__ void __launch_bounds__(THREADS) adjoint_agg_dpp_kernel(const BwdArgs a)
{
    constexpr int NGC = CHUNK_T / GROUP_T;
    __shared__ __attribute__((aligned(16))) float s_dt[ROWS][TPAD];
    __shared__ __attribute__((aligned(16))) float s_dy[ROWS][TPAD];
    __shared__ __attribute__((aligned(16))) float s_c[NGC][NPAD][GROUP_T];   // C of the chunk: [group][state][step]
    const FwdArgs& f = a.f;
    const int tid = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & (WAVE - 1);
    const int groups = (f.D + ROWS - 1) / ROWS;
    const unsigned bx = xcd_contiguous(blockIdx.x, gridDim.x);
    const int b = bx / groups;
    const int d0 = (bx % groups) * ROWS;
    const int L = f.L, N = f.N, NS = f.NS;
    const bool has_z = f.flags & F_HAS_Z, softplus = f.flags & F_DELTA_SOFTPLUS;
    const int seg = blockIdx.y + 1;  // segment 0 passes nothing on
    const int c_begin = seg * (f.seg_len / CHUNK_T);
    const int c_end = min((L + CHUNK_T - 1) / CHUNK_T, (seg + 1) * (f.seg_len / CHUNK_T));

    const int pr = pointwise_row_pitch9(tid), pq = tid & 3;   // TPAD = 36 floats
    const bool p_ok = d0 + pr < f.D;
    const int pd = p_ok ? d0 + pr : f.D - 1;
    const float bias = (f.flags & F_HAS_DELTA_BIAS) ? f.bias[pd] : 0.0f;
    const int rows_here = min(ROWS, f.D - d0);
    const long wg_first = ((long)b * f.D + d0) * L;
    const uint32_t wg_bytes = (uint32_t)rows_here * (uint32_t)L * (uint32_t)sizeof(T);
    const uint32_t row_off = (uint32_t)pr * (uint32_t)L * (uint32_t)sizeof(T);   // past the resource for rows past D
    const rsrc_t bd_ = make_rsrc(static_cast<const T*>(f.delta) + wg_first, wg_bytes);
    const rsrc_t bo_ = make_rsrc(static_cast<const T*>(a.dout) + wg_first, wg_bytes);
    const rsrc_t bz_ = make_rsrc(static_cast<const T*>(has_z ? f.z : f.delta) + wg_first, has_z ? wg_bytes : 0u);
    // staging view: waves 0, 1 stage C of the chunk; thread -> (state s_n, group of four steps s_tq)
    const int s_n = (tid >> 3) & (NPAD - 1), s_tq = tid & (NGC - 1);
    const rsrc_t bc_ = make_rsrc(static_cast<const T*>(f.Cm) + (long)b * f.bc_bstride,
                                 w < 2 ? (uint32_t)N * (uint32_t)L * (uint32_t)sizeof(T) : 0u);
    const uint32_t c_row_off = s_n < N ? (uint32_t)s_n * (uint32_t)L * (uint32_t)sizeof(T) : BUF_OFF;

    const bool s_ok = d0 + lane < f.D;
    const int sd = s_ok ? d0 + lane : f.D - 1;
    const long srow = (long)b * f.D + sd;
    float A2[STATES_PER_LANE], ag[STATES_PER_LANE];
#pragma unroll
    for (int k = 0; k < STATES_PER_LANE; ++k) {
        const int n = slot_state(w, k, f.il);
        const bool ok = n < N && k < SPL;
        A2[k] = (ok ? f.A[(long)sd * NS + n] : 0.0f) * LOG2E;
        ag[k] = (seg == f.nseg - 1 && ok && a.dh_last) ? a.dh_last[srow * NS + n] : 0.0f;
    }
    const int pat = slot_state(w, lane & 3, f.il);

    constexpr int PF = 2;
    typename io8<T>::raw rd_[PF], rz_[PF], ro_[PF];
    typename io4<T>::raw rc_[PF];
    auto issue_loads = [&](int c, auto slot_tag) {   // chunk c (walking down from c_end - 1) into a compile-time slot
        constexpr int s = decltype(slot_tag)::value;
        const int t0 = c * CHUNK_T + pq * SLICE;
        const uint32_t off = (t0 < L && c >= c_begin) ? row_off + (uint32_t)t0 * (uint32_t)sizeof(T) : BUF_OFF;   // slices are whole or empty
        rd_[s] = io8<T>::load_buf(bd_, off);
        ro_[s] = io8<T>::load_buf(bo_, off);
        rz_[s] = io8<T>::load_buf(bz_, off);
        const int ts = c * CHUNK_T + s_tq * GROUP_T;
        rc_[s] = io4<T>::load_buf(bc_, (ts < L && c >= c_begin) ? c_row_off + (uint32_t)ts * (uint32_t)sizeof(T) : BUF_OFF);
    };
    issue_loads(c_end - 1, std::integral_constant<int, 0>{});
    issue_loads(c_end - 2, std::integral_constant<int, 1>{});

    auto do_chunk = [&](const int c, auto slot_tag) {
        constexpr int SLOT = decltype(slot_tag)::value;
        const int t0 = c * CHUNK_T + pq * SLICE;
        const bool live = p_ok && t0 < L;
        {
            float v8[SLICE], o8[SLICE], z8[SLICE], dt8[SLICE], c4[GROUP_T];
            io8<T>::unpack(rd_[SLOT], v8);
            io8<T>::unpack(ro_[SLOT], o8);
            if (has_z) io8<T>::unpack(rz_[SLOT], z8);
            io4<T>::unpack(rc_[SLOT], c4);
            const float bias_eff = live ? bias : (softplus ? -1e30f : 0.0f);   // an empty slice runs with dt = 0
#pragma unroll
            for (int j = 0; j < SLICE; ++j) {
                const float x = v8[j] + bias_eff;
                float sp, sg;
                if (softplus) softplus_sigmoid(x, sp, sg); else sp = x;
                dt8[j] = sp;
                if (has_z) o8[j] *= z8[j] * sigmoid_fast(z8[j]);
            }
            float4* pd4 = reinterpret_cast<float4*>(&s_dt[pr][pq * SLICE]);
            float4* py4 = reinterpret_cast<float4*>(&s_dy[pr][pq * SLICE]);
            pd4[0] = make_float4(dt8[0], dt8[1], dt8[2], dt8[3]);
            pd4[1] = make_float4(dt8[4], dt8[5], dt8[6], dt8[7]);
            py4[0] = make_float4(o8[0], o8[1], o8[2], o8[3]);
            py4[1] = make_float4(o8[4], o8[5], o8[6], o8[7]);
            if (w < 2) *reinterpret_cast<float4*>(&s_c[s_tq][s_n][0]) = make_float4(c4[0], c4[1], c4[2], c4[3]);
        }
        issue_loads(c - PF, slot_tag);
        __syncthreads();
        __builtin_amdgcn_s_setprio(2);   // as in scan_bwd_kernel: the recurrence at a raised wave priority
        float4 dtc[NGC], dyc[NGC], Cpc[NGC];
#pragma unroll
        for (int g = 0; g < NGC; ++g) {
            dtc[g] = *reinterpret_cast<const float4*>(&s_dt[lane][g * GROUP_T]);
            dyc[g] = *reinterpret_cast<const float4*>(&s_dy[lane][g * GROUP_T]);
            Cpc[g] = *reinterpret_cast<const float4*>(&s_c[g][pat][0]);
        }
#pragma unroll
        for (int g = NGC - 1; g >= 0; --g) {
#pragma unroll
            for (int j = GROUP_T - 1; j >= 0; --j) {
                const float dt = f4_get(dtc[g], j), dy = f4_get(dyc[g], j);
                adjoint_input_dpp<SPL>(ag, f4_get(Cpc[g], j), dy);          // g = C dy + abar+ g+
#pragma unroll
                for (int k = 0; k < SPL; ++k) ag[k] *= exp2_fast(dt * A2[k]);   // flows on to h_{t-1}
            }
        }
        __builtin_amdgcn_s_setprio(0);
        __syncthreads();
    };
    for (int c = c_end - 1; c >= c_begin; c -= PF) {
        do_chunk(c, std::integral_constant<int, 0>{});
        if (c - 1 >= c_begin) do_chunk(c - 1, std::integral_constant<int, 1>{});
    }
    if (s_ok) {
        float4* dst = reinterpret_cast<float4*>(a.seg_g + ((long)seg * f.B * f.D + srow) * NPAD) + w;
        *dst = make_float4(ag[0], ag[1], ag[2], ag[3]);
    }
}

// Turns the segments' local adjoint carries into incoming ones, in place, walking the
// segments backwards: in[nseg-2] = loc[nseg-1];  in[s-1] = exp(A * sum_dt[s]) * in[s] + loc[s].
__global__ void carry_bwd_kernel(const BwdArgs a)
{
    const FwdArgs& f = a.f;
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const long rows = (long)f.B * f.D;
    if (i >= rows * NPAD) return;
    const long row = i / NPAD;
    const int n = position_state((int)(i % NPAD), f.il), d = row % f.D;   // the state this slot of the record holds
    const float A2 = n < f.N ? f.A[(long)d * f.NS + n] * LOG2E : 0.0f;
    // complex state: slots (n, n^1) are one state; the carry is multiplied by conj(exp(A sum_dt))
    const bool cplx_state = f.flags & F_COMPLEX;
    const long ip = i ^ 1;
    const float A2r = cplx_state && (n & ~1) < f.N ? f.A[(long)d * f.NS + (n & ~1)] * LOG2E : 0.0f;
    const float Aim = cplx_state && (n | 1) < f.N ? f.A[(long)d * f.NS + (n | 1)] : 0.0f;
    float carry = a.seg_g[(long)(f.nseg - 1) * rows * NPAD + i];  // loc of the last segment (includes dh_last)
    float other = cplx_state ? a.seg_g[(long)(f.nseg - 1) * rows * NPAD + ip] : 0.0f;
    // as in carry_fwd_kernel: loads of a batch of segments first, then the serial chain
    constexpr int CARRY_BATCH = 16;
    for (int s0 = f.nseg - 2; s0 >= 0; s0 -= CARRY_BATCH) {
        float loc[CARRY_BATCH], locp[CARRY_BATCH], sdt[CARRY_BATCH];
#pragma unroll
        for (int j = 0; j < CARRY_BATCH; ++j) {
            const int s = s0 - j;
            loc[j] = s >= 1 ? a.seg_g[(long)s * rows * NPAD + i] : 0.0f;   // segment 0 has no aggregate
            locp[j] = (cplx_state && s >= 1) ? a.seg_g[(long)s * rows * NPAD + ip] : 0.0f;
            sdt[j] = s >= 1 ? f.seg_sumdt[(long)s * rows + row] : 0.0f;
        }
#pragma unroll
        for (int j = 0; j < CARRY_BATCH; ++j) {
            const int s = s0 - j;
            if (s >= 0) {
                a.seg_g[(long)s * rows * NPAD + i] = carry;  // carry entering segment s from the right
                if (cplx_state) {
                    const cplx ab = complex_decay(sdt[j], A2r, Aim);
                    const float re = (n & 1) ? other : carry, im = (n & 1) ? carry : other;
                    const float nre = fmaf(ab.re, re, ab.im * im) + ((n & 1) ? locp[j] : loc[j]);
                    const float nim = fmaf(ab.re, im, -ab.im * re) + ((n & 1) ? loc[j] : locp[j]);
                    carry = (n & 1) ? nim : nre;
                    other = (n & 1) ? nre : nim;
                } else {
                    carry = fmaf(exp2_fast(A2 * sdt[j]), carry, loc[j]);
                }
            }
        }
    }
}

// dB and dC are accumulated atomically by the scan kernel and must start at zero (a null
// pointer: that gradient belongs to a time-invariant operand and is written elsewhere).
__global__ void zero_kernel(float* __restrict__ p0, float* __restrict__ p1, long n)
{
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        if (p0) p0[i] = 0.0f;
        if (p1) p1[i] = 0.0f;
    }
}

// Sum the per-batch partials: dA (D,N), dD (D), dbias (D).  With L == 0 (no partials
// written) everything is zero.
__global__ void finalize_kernel(const BwdArgs a, int have_partials)
{
    const int d = blockIdx.x * blockDim.x / NPAD + threadIdx.x / NPAD;
    const int n = threadIdx.x % NPAD;
    if (d >= a.f.D) return;
    float sA = 0.0f, sD = 0.0f, sb = 0.0f, sB = 0.0f, sC = 0.0f;
    const bool bfix = a.f.flags & F_B_FIXED, cfix = a.f.flags & F_C_FIXED;
    if (have_partials) {
#pragma unroll 8
        for (int b = 0; b < a.f.B * a.f.nseg; ++b) {  // per segment and batch entry
            const long row = (long)b * a.f.D + d;
            sA += a.dA_part[row * NPAD + n];
            if (bfix) sB += a.dBf_part[row * NPAD + n];   // time-invariant B / C are never split: nseg == 1
            if (cfix) sC += a.dCf_part[row * NPAD + n];
            if (n == 0) { sD += a.dD_part[row]; sb += a.db_part[row]; }
        }
    }
    const int st = position_state(n, a.f.il);   // the state whose partial sums sit at slot n of the records
    if (st < a.f.N) a.dA[(long)d * a.f.NS + st] = sA;
    if (st < a.f.N && bfix) a.dB[(long)d * a.f.NS + st] = sB;
    if (st < a.f.N && cfix) a.dC[(long)d * a.f.NS + st] = sC;
    if (n == 0) {
        if (a.dD) a.dD[d] = sD;   // null for all but the first state group
        if (a.dbias) a.dbias[d] = a.acc ? a.dbias[d] + sb : sb;
    }
}

__global__ void copy_dh_kernel(const float* __restrict__ src, float* __restrict__ dst, long n)
{
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src ? src[i] : 0.0f;
}

// The backward kernel's LDS tiles exceed the default dynamic limit; raising it is needed once per
// kernel and per device; `done` is the calling launcher's table for its kernel, indexed by device.
constexpr int MAX_DEVICES = 64;
template <typename K>
static bool allow_backward_lds_once(K kern, std::atomic<bool> (&done)[MAX_DEVICES], size_t bytes)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return false;
    if (done[dev].load(std::memory_order_acquire)) return true;
    if (hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess)
        return false;   // setting it twice from two threads is harmless
    done[dev].store(true, std::memory_order_release);
    return true;
}

template <typename T, bool VEC, bool FULLN, bool ZOH, int BCFIX>
static int launch_scan_bwd_fixed(const BwdArgs& a, dim3 grid, hipStream_t stream)
{
    auto kern = scan_bwd_kernel<T, VEC, FULLN, ZOH, BCFIX>;
    static std::atomic<bool> lds_ok[MAX_DEVICES];   // this launcher is instantiated once per kernel
    if (!allow_backward_lds_once(reinterpret_cast<const void*>(kern), lds_ok, sizeof(BwdSmem))) return -1;
    kern<<<dim3(grid.x, 1u), dim3(THREADS), sizeof(BwdSmem), stream>>>(a);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// complex state: first-order B-bar only; selective or time-invariant B / C
template <typename T, bool VEC, bool FULLN, int BCFIX>
static int launch_scan_bwd_complex(const BwdArgs& a, dim3 grid, hipStream_t stream)
{
    auto kern = scan_bwd_kernel<T, VEC, FULLN, false, BCFIX, true>;
    static std::atomic<bool> lds_ok[MAX_DEVICES];   // this launcher is instantiated once per kernel
    if (!allow_backward_lds_once(reinterpret_cast<const void*>(kern), lds_ok, sizeof(BwdSmem))) return -1;
    if (a.f.nseg > 1) {   // only with selective B and C (the planner does not split the others)
        adjoint_agg_kernel<T, VEC, FULLN, true><<<dim3(grid.x, (unsigned)(a.f.nseg - 1)), dim3(THREADS), 0, stream>>>(a);
        const long n = (long)a.f.B * a.f.D * NPAD;
        carry_bwd_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream>>>(a);
    }
    kern<<<dim3(grid.x, (unsigned)a.f.nseg), dim3(THREADS), sizeof(BwdSmem), stream>>>(a);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// the common case (scan_bwd_dpp_kernel), with the adjoint aggregates of a split sequence first
template <typename T, bool FULLN, int SPL, bool ZOH = false>
static int launch_scan_bwd_dpp(const BwdArgs& a, dim3 grid, hipStream_t stream)
{
    if (a.f.nseg > 1) {
        adjoint_agg_dpp_kernel<T, SPL><<<dim3(grid.x, (unsigned)(a.f.nseg - 1)), dim3(THREADS), 0, stream>>>(a);
        const long n = (long)a.f.B * a.f.D * NPAD;
        carry_bwd_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream>>>(a);
    }
    auto kern = scan_bwd_dpp_kernel<T, SPL, ZOH>;
    static std::atomic<bool> lds_ok[MAX_DEVICES];   // this launcher is instantiated once per kernel
    if (!allow_backward_lds_once(reinterpret_cast<const void*>(kern), lds_ok, sizeof(BwdSmemDpp))) return -1;
    kern<<<dim3(grid.x, (unsigned)a.f.nseg), dim3(THREADS), sizeof(BwdSmemDpp), stream>>>(a);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

template <typename T, bool VEC, bool FULLN, bool ZOH>
static int launch_scan_bwd(const BwdArgs& a, dim3 grid, hipStream_t stream)
{
    const int bcfix = ((a.f.flags & F_B_FIXED) ? 1 : 0) | ((a.f.flags & F_C_FIXED) ? 2 : 0);
    if constexpr (!ZOH) {
        if (a.f.flags & F_COMPLEX) {
            if (bcfix == 0) return launch_scan_bwd_complex<T, VEC, FULLN, 0>(a, grid, stream);
            if (bcfix == 1) return launch_scan_bwd_complex<T, VEC, FULLN, 1>(a, grid, stream);
            if (bcfix == 2) return launch_scan_bwd_complex<T, VEC, FULLN, 2>(a, grid, stream);
            return launch_scan_bwd_complex<T, VEC, FULLN, 3>(a, grid, stream);
        }
    }
    if (bcfix == 1) return launch_scan_bwd_fixed<T, VEC, FULLN, ZOH, 1>(a, grid, stream);
    if (bcfix == 2) return launch_scan_bwd_fixed<T, VEC, FULLN, ZOH, 2>(a, grid, stream);
    if (bcfix == 3) return launch_scan_bwd_fixed<T, VEC, FULLN, ZOH, 3>(a, grid, stream);
    if constexpr (VEC && FULLN && ZOH) {   // exact ZOH: the same kernel, built for sixteen states
        return launch_scan_bwd_dpp<T, FULLN, STATES_PER_LANE, true>(a, grid, stream);
    } else if constexpr (VEC && !ZOH) {   // real state, first-order B-bar, selective B and C, whole 16-byte pieces
        if constexpr (!FULLN) {    // fewer than 16 states dealt out to the waves: kernels built for 1 or 2 slots per lane
            const int spl = slots_for(a.f.N, a.f.il);
            if (spl == 1) return launch_scan_bwd_dpp<T, FULLN, 1>(a, grid, stream);
            if (spl == 2) return launch_scan_bwd_dpp<T, FULLN, 2>(a, grid, stream);
        }
        return launch_scan_bwd_dpp<T, FULLN, STATES_PER_LANE>(a, grid, stream);
    } else {
        if (a.f.nseg > 1) {
            adjoint_agg_kernel<T, VEC, FULLN><<<dim3(grid.x, (unsigned)(a.f.nseg - 1)), dim3(THREADS), 0, stream>>>(a);
            const long n = (long)a.f.B * a.f.D * NPAD;
            carry_bwd_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream>>>(a);
        }
        auto kern = scan_bwd_kernel<T, VEC, FULLN, ZOH>;
        static std::atomic<bool> lds_ok[MAX_DEVICES];   // this launcher is instantiated once per kernel
        if (!allow_backward_lds_once(reinterpret_cast<const void*>(kern), lds_ok, sizeof(BwdSmem))) return -1;
        kern<<<dim3(grid.x, (unsigned)a.f.nseg), dim3(THREADS), sizeof(BwdSmem), stream>>>(a);
        return hipGetLastError() == hipSuccess ? 0 : -1;
    }
}

int launch_bwd(const BwdArgs& a, int io_dtype, hipStream_t stream)
{
    const FwdArgs& f = a.f;
    const int fin_blocks = (f.D * NPAD + 255) / 256;
    if (f.L == 0) {
        finalize_kernel<<<dim3(fin_blocks), dim3(256), 0, stream>>>(a, 0);
        if (a.dh0 && !a.acc) {
            const long n = (long)f.B * f.D * f.NS;
            copy_dh_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream>>>(a.dh_last, a.dh0, n);
        }
        return hipGetLastError() == hipSuccess ? 0 : -1;
    }
    // the first state group clears dB and dC for all of them
    const long nbc = (long)f.B * f.NS * f.L;
    float* const zB = ((f.flags & F_B_FIXED) || a.acc) ? nullptr : a.dB;
    float* const zC = ((f.flags & F_C_FIXED) || a.acc) ? nullptr : a.dC;
    if (zB || zC) zero_kernel<<<dim3((unsigned)((nbc + 255) / 256)), dim3(256), 0, stream>>>(zB, zC, nbc);
    const int groups = (f.D + ROWS - 1) / ROWS;
    const dim3 grid((unsigned)(f.B * groups));
    const bool fulln = f.N == NPAD;
    int rc;
    if (f.flags & F_EXACT_ZOH_B) {  // the variant is built for the fastest and the most general shape only
        if (io_dtype == 0) {
            if (f.vec_ok && fulln) rc = launch_scan_bwd<float, true, true, true>(a, grid, stream);
            else rc = launch_scan_bwd<float, false, false, true>(a, grid, stream);
        } else {
            if (f.vec_ok && fulln) rc = launch_scan_bwd<bf16_t, true, true, true>(a, grid, stream);
            else rc = launch_scan_bwd<bf16_t, false, false, true>(a, grid, stream);
        }
    } else if (io_dtype == 0) {
        if (f.vec_ok && fulln) rc = launch_scan_bwd<float, true, true, false>(a, grid, stream);
        else if (f.vec_ok) rc = launch_scan_bwd<float, true, false, false>(a, grid, stream);
        else rc = launch_scan_bwd<float, false, false, false>(a, grid, stream);
    } else {
        if (f.vec_ok && fulln) rc = launch_scan_bwd<bf16_t, true, true, false>(a, grid, stream);
        else if (f.vec_ok) rc = launch_scan_bwd<bf16_t, true, false, false>(a, grid, stream);
        else rc = launch_scan_bwd<bf16_t, false, false, false>(a, grid, stream);
    }
    if (rc != 0) return rc;
    finalize_kernel<<<dim3(fin_blocks), dim3(256), 0, stream>>>(a, 1);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // namespace ss
