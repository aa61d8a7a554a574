// Forward selective scan (Algorithm 2 steps 5-6, fused as in Appendix D "Speed") and the
// single-token recurrent step (Section 2, Eq. 2a/2b applied once).
#include <type_traits>

#include "ss_kernels.h"
#include "ss_device.h"

namespace ss {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));   // MFMA operand and accumulator types

// One workgroup = 64 rows x 4 waves.  Per chunk of CHUNK_T steps:
//   A. (pointwise view) load 64 rows x 32 steps of u, delta, z with 16-byte accesses, form
//      dt = softplus(delta + bias) and dt*u, park them in LDS;
//   B. (state view) wave w runs Eq. 2a/2b sequentially over the 32 steps for states
//      4w..4w+3 of its 64 rows, B and C arriving as scalar operands, and writes its
//      partial sum over those states of C*h to LDS;
//   C. (pointwise view) add the 4 partial sums, the skip term and the gate, and store.
// The state never leaves registers between chunks (Appendix D: the scan continues from
// the previous chunk's state).  Steps past the end of the sequence use dt = 0, which is
// the identity of the recurrence (abar = 1, input term 0).
//
// When the sequence is split into segments (blockIdx.y), the kernel runs twice: first with
// AGG = true on every segment but the last, from the zero state (segment 0: from h0),
// producing only the segment's end state and the sum of its step sizes; then, after
// carry_fwd_kernel has turned those into each segment's incoming state, with AGG = false.
// ZOH selects the exact zero-order-hold B-bar of Eq. 4: the LDS tile that otherwise carries
// dt*u then carries u, and each state multiplies it by phi(dt, A) = (abar - 1) / A.
// BCFIX: bit 0 / bit 1 set when B / C is the time-invariant (D,N) float32 parameter of
// Algorithm 1 instead of the selective (B,N,L) tensor: it then sits in registers like A.
// CPLX: the lane's four state slots are two complex states (re, im) each (Section 3.6); only
// the recurrence and the read-out differ, everything around them sees 2N real "states".
// STAGED: B and C come from the wave-packed copy a.bcs that stage_bc_kernel made: one scalar
// load per group instead of eight, one address per wave instead of eight clamped ones, so the
// scalar registers suffice for a whole group of prefetch and the scalar unit does little but
// widen bf16.  (Read in place, the eight loads of the next group compete with the current
// group's operands for scalar registers, some are issued only right before their use, and the
// wait for those drains the whole prefetch: the loads' latency shows once per group.)
// FUSED_KS > 0 (bf16, VEC, STAGED, main pass of an unsplit sequence): delta_raw = W_dt r is not
// read but formed here, per chunk, as a 64 x 32 product over R <= 32 * FUSED_KS on the matrix
// cores: wave w owns rows 16w..16w+15 (its pieces of W_dt stay in registers for the whole
// kernel) and both 16-step halves of the chunk; the result goes through the dt tile in LDS to
// the pointwise threads, rounded to bf16 as the stored delta would be.  Saves the projection
// kernel and the write and read of a (B,D,L) tensor.
// SPL: slots per lane the recurrence is built for (4, or ceil(N / 4) rounded up to 1 or 2 when the
// states are dealt out to the waves in turn, FwdArgs::il).
// PAT (VEC, real state, selective B and C): B and C take neither scalar path.  The chunk's B and C are
// requested with the chunk's u, delta and z by ordinary buffer loads (thread -> B or C, state, group
// of four steps), widened to float and put into an LDS tile [group][state][step]; lane l of wave w
// reads, per group, one float4 with the state of slot l % 4 at the group's four steps, and the
// recurrence takes a state's value from that register as a quad-broadcast DPP operand
// (input_step_dpp, readout_step_dpp).  No scalar loads or their waits (which also drain LDS reads and
// vice versa), no repacking pass, no touching of cache lines ahead, and no vector-memory wait that
// has to cover the previous chunk's stores.
template <typename T, bool VEC, bool FULLN, bool AGG, bool ZOH, int BCFIX = 0, bool CPLX = false, bool STAGED = false,
          int FUSED_KS = 0, int SPL = STATES_PER_LANE, bool PAT = false>
__global__ void __launch_bounds__(THREADS, (PAT && FUSED_KS <= 4 && !(ZOH && AGG)) ? 2 : 1) scan_fwd_kernel(const FwdArgs a)
{
    static_assert(!PAT || (VEC && BCFIX == 0 && !CPLX && !STAGED), "PAT: vector path, real state, selective B and C");
    constexpr int NGC = CHUNK_T / GROUP_T;
    __shared__ __attribute__((aligned(16))) float s_bc[PAT ? 2 : 1][PAT ? NGC : 1][PAT ? NPAD : 1][GROUP_T];   // PAT: B (0) and C (1) of the chunk
    __shared__ __attribute__((aligned(16))) float s_dt[ROWS][TPAD];
    __shared__ __attribute__((aligned(16))) float s_du[ROWS][TPAD];
    __shared__ __attribute__((aligned(16))) float s_yp[NWAVES][ROWS][TPAD];
    __shared__ __attribute__((aligned(16))) float s_raw[FUSED_KS > 0 ? ROWS : 1][TPAD];   // FUSED: delta_raw of the next chunk
    constexpr int RT_PITCH = 32 * (FUSED_KS > 0 ? FUSED_KS : 1) + 8;                     // bf16 elements; rows 16 bytes off the banks
    __shared__ __attribute__((aligned(16))) bf16_t s_rT[FUSED_KS > 0 ? CHUNK_T : 1][RT_PITCH];   // FUSED: r of the next chunk's steps

    const int tid = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave index, provably uniform
    const int lane = tid & (WAVE - 1);
    const int groups = (a.D + ROWS - 1) / ROWS;
    // Workgroups go to the eight XCDs in turn by index; with this renumbering each XCD gets a contiguous
    // run of row groups, i.e. one batch entry's rows, whose shared operands (B, C, r) then meet in its L2.
    const unsigned bx = xcd_contiguous(blockIdx.x, gridDim.x);
    const int b = bx / groups;
    const int d0 = (bx % groups) * ROWS;
    const int L = a.L, N = a.N, NS = a.NS;
    const bool has_z = !AGG && (a.flags & F_HAS_Z), has_D = !AGG && (a.flags & F_HAS_D);
    const bool softplus = a.flags & F_DELTA_SOFTPLUS;
    const int seg = blockIdx.y;
    const int c_begin = seg * (a.seg_len / CHUNK_T);
    const int c_end = min((L + CHUNK_T - 1) / CHUNK_T, (seg + 1) * (a.seg_len / CHUNK_T));

    // ---- pointwise view: thread -> (row pr, slice pq) -----------------------------------
    const int pr = pointwise_row_pitch9(tid), pq = tid & 3;   // TPAD = 36 floats
    const bool p_ok = d0 + pr < a.D;
    const int pd = p_ok ? d0 + pr : a.D - 1;  // out-of-range rows shadow the last row; stores masked
    const long prow = (long)b * a.D + pd;
    const T* __restrict__ gu = static_cast<const T*>(a.u) + prow * L;
    const T* __restrict__ gdl = static_cast<const T*>(a.delta) + prow * L;
    const T* __restrict__ gz = static_cast<const T*>(a.z) + prow * L;  // not dereferenced without z
    T* __restrict__ gout = static_cast<T*>(a.out) + prow * L;
    const float bias = (a.flags & F_HAS_DELTA_BIAS) ? a.bias[pd] : 0.0f;
    const float Dsk = has_D ? a.Dskip[pd] : 0.0f;
    // VEC: buffer resources over this workgroup's rows of each tensor (a size of zero switches
    // an optional tensor off), so that the accesses in the loop are issued unconditionally
    const int rows_here = min(ROWS, a.D - d0);
    const long wg_first = ((long)b * a.D + d0) * L;
    const uint32_t wg_bytes = (uint32_t)rows_here * (uint32_t)L * (uint32_t)sizeof(T);
    const uint32_t row_off = (uint32_t)pr * (uint32_t)L * (uint32_t)sizeof(T);   // past the resource for rows past D
    const bool keep_y = !AGG && has_z && a.ysave;
    const rsrc_t bu = make_rsrc(static_cast<const T*>(a.u) + wg_first, wg_bytes);
    const rsrc_t bd = make_rsrc(static_cast<const T*>(a.delta) + wg_first, wg_bytes);
    const rsrc_t bz = make_rsrc(static_cast<const T*>(has_z ? a.z : a.u) + wg_first, has_z ? wg_bytes : 0u);
    const rsrc_t bo = make_rsrc(static_cast<T*>(AGG ? const_cast<void*>(a.u) : a.out) + wg_first, AGG ? 0u : wg_bytes);
    const rsrc_t by = make_rsrc(static_cast<T*>(keep_y ? a.ysave : const_cast<void*>(a.u)) + wg_first, keep_y ? wg_bytes : 0u);
    // what the earlier state groups left (more than 16 states): prefetched like an input, so that no wait in the loop has to drain the memory pipeline
    const bool acc_on = !AGG && a.acc_y;
    const rsrc_t bp = make_rsrc(static_cast<const T*>(acc_on ? (has_z ? a.ysave : a.out) : a.u) + wg_first, acc_on ? wg_bytes : 0u);
    // PAT staging view: waves 0, 1 stage B, waves 2, 3 stage C (not needed for the aggregates);
    // thread -> (state s_n, group of four steps s_tq) of the chunk
    const int s_which = w >> 1, s_n = (tid >> 3) & (NPAD - 1), s_tq = tid & (NGC - 1);
    const bool s_on = PAT && !(AGG && s_which == 1);
    const rsrc_t bbc = make_rsrc(static_cast<const T*>(s_which ? a.Cm : a.Bm) + (long)b * a.bc_bstride,
                                 s_on ? (uint32_t)N * (uint32_t)L * (uint32_t)sizeof(T) : 0u);
    const uint32_t bc_row_off = s_n < N ? (uint32_t)s_n * (uint32_t)L * (uint32_t)sizeof(T) : BUF_OFF;

    // ---- state view: lane -> row, wave -> states 4w..4w+3 -------------------------------
    const bool s_ok = d0 + lane < a.D;
    const int sd = s_ok ? d0 + lane : a.D - 1;
    const long srow = (long)b * a.D + sd;
    constexpr bool BFIX = BCFIX & 1, CFIX = BCFIX & 2;
    float A2[STATES_PER_LANE], An[STATES_PER_LANE], invA[STATES_PER_LANE], h[STATES_PER_LANE];
    float Bf[STATES_PER_LANE], Cf[STATES_PER_LANE];
    const T* __restrict__ gB[STATES_PER_LANE];
    const T* __restrict__ gC[STATES_PER_LANE];
    bool n_ok[STATES_PER_LANE];
#pragma unroll
    for (int k = 0; k < STATES_PER_LANE; ++k) {
        const int n = slot_state(w, k, a.il);
        n_ok[k] = n < N && k < SPL;
        const int nc = n_ok[k] ? n : 0;
        An[k] = n_ok[k] ? a.A[(long)sd * NS + nc] : 0.0f;
        A2[k] = An[k] * LOG2E;
        invA[k] = An[k] != 0.0f ? 1.0f / An[k] : 0.0f;
        if (seg == 0) h[k] = (n_ok[k] && (a.flags & F_HAS_H0)) ? a.h0[srow * NS + nc] : 0.0f;
        else h[k] = AGG ? 0.0f : a.seg_h[((long)seg * a.B * a.D + srow) * NPAD + w * STATES_PER_LANE + k];
        gB[k] = BFIX ? nullptr : static_cast<const T*>(a.Bm) + (long)b * a.bc_bstride + (long)nc * L;
        gC[k] = CFIX ? nullptr : static_cast<const T*>(a.Cm) + (long)b * a.bc_bstride + (long)nc * L;
        Bf[k] = (BFIX && n_ok[k]) ? static_cast<const float*>(a.Bm)[(long)sd * NS + nc] : 0.0f;
        Cf[k] = (CFIX && n_ok[k]) ? static_cast<const float*>(a.Cm)[(long)sd * NS + nc] : 0.0f;
    }
    // staged B and C: this wave's pieces, one per group of steps, consecutive in memory
    const T* __restrict__ const sbc =
        STAGED ? static_cast<const T*>(a.bcs) + (((long)b * ((NS + NPAD - 1) / NPAD * NWAVES) + w) * (a.Lp / GROUP_T)) * STAGE_GROUP
               : nullptr;
    // the selective operands (if any) whose cache lines are touched one chunk ahead
    const void* const touchB = BFIX ? a.Cm : a.Bm;
    const void* const touchC = CFIX ? a.Bm : a.Cm;
    // staged: the wave's pieces of a chunk are contiguous; a lane touches every 16th element
    const rsrc_t bt = make_rsrc(sbc, STAGED ? (uint32_t)(a.Lp / GROUP_T) * STAGE_GROUP * (uint32_t)sizeof(T) : 0u);
    auto touch = [&](int t) -> uint32_t {
        if constexpr (STAGED) {   // an unconditional buffer load; lanes with nothing to touch are out of range
            constexpr int per_chunk = CHUNK_T / GROUP_T * STAGE_GROUP;
            const bool on = lane * 16 < per_chunk && t >= 0 && t < a.Lp;
            const uint32_t off = on ? (uint32_t)((t / GROUP_T) * STAGE_GROUP + lane * 16) * (uint32_t)sizeof(T) : BUF_OFF;
            return (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(bt, (int)off, 0, 0);
        } else {
            return touch_bc<T>(touchB, touchC, b, a.bc_bstride, N, L, w, lane, t);
        }
    };
    float sum_dt = 0.0f;  // AGG: this thread's share of the segment's sum of step sizes

    // FUSED: operand fragments of the 16x16x32 bf16 MFMA.  Lane l holds row (column) l % 16 of
    // the first (second) operand at contraction indices 8 * (l / 16) ..+7 of each 32-wide step;
    // accumulator element i of lane l is row 4 * (l / 16) + i, column l % 16.
    constexpr int KS = FUSED_KS > 0 ? FUSED_KS : 1;
    union Frag { unsigned short s[8]; bf16x8_t v; };
    Frag wfr[KS];
    constexpr int RLD = (KS + 1) / 2;          // 16-byte pieces of the chunk's r per thread: 32 steps x Rp / 256 threads
    Frag rld[RLD];
    const int fsub = 8 * (lane >> 4);
    const int rt_t = tid >> 3, rt_col = (tid & 7) * 4 * KS;   // this thread's piece of the (32 steps, Rp) tile
    if constexpr (FUSED_KS > 0) {
        const bf16_t* wp = static_cast<const bf16_t*>(a.W_dt) + (long)min(d0 + 16 * w + (lane & 15), a.D - 1) * a.R;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int k = 32 * ks + fsub;
            wfr[ks].v = *reinterpret_cast<const bf16x8_t*>(wp + min(k, a.R - 8));   // R is a multiple of 8
            if (k >= a.R) {
#pragma unroll
                for (int e = 0; e < 8; ++e) wfr[ks].s[e] = 0;
            }
        }
    }
    // u, delta and z are requested PF chunks ahead (slot = chunk index mod PF): the scan is not long
    // enough to cover a memory round trip under load, and with one chunk in flight per workgroup
    // the kernel ran at the pace of that latency whatever the state size.
    constexpr int PF = VEC ? 2 : 1;
    typename io8<T>::raw ru_[PF], rd_[PF], rz_[PF];
    typename io4<T>::raw rbc_[PF];   // PAT: the thread's four steps of B or C
    typename io8<T>::raw rp_[PF];    // VEC: the pre-gate y of the earlier state groups (zeros if there are none)
    auto issue_loads = [&](int c, auto slot_tag) {   // chunk c into the slot given at compile time
        constexpr int s = decltype(slot_tag)::value;
        const int t0 = c * CHUNK_T + pq * SLICE;
        const int nv = min(max(L - t0, 0), SLICE);
        if constexpr (VEC) {   // slices are whole or empty
            const uint32_t off = (nv == SLICE && c < c_end) ? row_off + (uint32_t)t0 * (uint32_t)sizeof(T) : BUF_OFF;
            ru_[s] = io8<T>::load_buf(bu, off);
            if constexpr (FUSED_KS == 0) rd_[s] = io8<T>::load_buf(bd, off);
            rz_[s] = io8<T>::load_buf(bz, off);
            rp_[s] = io8<T>::load_buf(bp, off);
            if constexpr (PAT) {   // L % 8 == 0: a group of four steps is whole or past the end
                const int ts = c * CHUNK_T + s_tq * GROUP_T;
                rbc_[s] = io4<T>::load_buf(bbc, (ts < L && c < c_end) ? bc_row_off + (uint32_t)ts * (uint32_t)sizeof(T) : BUF_OFF);
            }
        } else {
            ru_[s] = io8<T>::template load<VEC>(gu + t0, nv);
            rd_[s] = io8<T>::template load<VEC>(gdl + t0, nv);
            if (has_z) rz_[s] = io8<T>::template load<VEC>(gz + t0, nv);
        }
    };
    // FUSED: delta_raw of a chunk from the fragments in registers: two 16 x 16 tiles per wave,
    // into rows 16w..16w+15 of s_raw -- the rows this wave's own pointwise threads read, so the
    // exchange needs no workgroup barrier (a wave's LDS instructions execute in order).  Called
    // for the next chunk after the recurrence, where the matrix-core latency hides behind the
    // pointwise post-processing.
    auto project = [&]() {
        if constexpr (FUSED_KS > 0) {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");   // earlier reads of s_raw are done
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) {
                f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
                    if (32 * ks < a.Rp) {
                        const bf16x8_t rv = *reinterpret_cast<const bf16x8_t*>(&s_rT[16 * nt + (lane & 15)][32 * ks + fsub]);
                        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wfr[ks].v, rv, acc, 0, 0, 0);
                    }
#pragma unroll
                for (int i = 0; i < 4; ++i) s_raw[16 * w + 4 * (lane >> 4) + i][16 * nt + (lane & 15)] = acc[i];
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
    };
    // FUSED: r of a chunk's 32 steps (transposed and padded, so always in range) is read once per
    // workgroup, two chunks ahead into registers, one chunk ahead into LDS
    auto issue_r = [&](int c) {
        if constexpr (FUSED_KS > 0) {
            const bf16_t* rp = static_cast<const bf16_t*>(a.rT) + ((long)b * a.Lp + min(max(c, 0) * CHUNK_T, a.Lp - CHUNK_T) + rt_t) * a.Rp;
#pragma unroll
            for (int j = 0; j < RLD; ++j)
                rld[j].v = *reinterpret_cast<const bf16x8_t*>(rp + min(rt_col + 8 * j, a.Rp - 8));
        }
    };
    auto stage_r = [&]() {   // this thread's piece of the chunk's r, from registers to LDS
        if constexpr (FUSED_KS > 0) {
#pragma unroll
            for (int j = 0; j < RLD; ++j)
                if (rt_col + 8 * j < a.Rp) *reinterpret_cast<bf16x8_t*>(&s_rT[rt_t][rt_col + 8 * j]) = rld[j].v;
        }
    };
    // The wait the compiler puts before a chunk's first use of its inputs allows as many memory
    // operations in flight as the shortest path into that point issues after them.  The way in from
    // here must not be that path, or every iteration would drain the stores it has just issued: the
    // first chunk's requests go out first and stay in that order.
    issue_loads(c_begin, std::integral_constant<int, 0>{});
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (PF > 1) issue_loads(c_begin + 1, std::integral_constant<int, 1>{});
    __builtin_amdgcn_sched_barrier(0);
    // PAIR (16-bit elements): a 32-step chunk is 64 bytes of a row, half a 128-byte line.  Writes of
    // half lines reach about half the throughput of whole lines (and reads somewhat less than whole
    // ones), so the traffic of an even chunk and the odd one after it (segments start at even
    // chunks) is issued together: both chunks' inputs are requested in the odd chunk's phase A, tensor
    // by tensor, and the even chunk's results wait in registers for the odd chunk's.
    constexpr bool PAIR = PAT && sizeof(T) == 2 && PF == 2;
    auto issue_pair = [&](int c0) {   // chunks c0 (slot 0) and c0 + 1 (slot 1)
      if constexpr (PAIR) {
        uint32_t off[2], boff[2];
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int c = c0 + s;
            const int t0 = c * CHUNK_T + pq * SLICE;
            off[s] = (t0 + SLICE <= L && c < c_end) ? row_off + (uint32_t)t0 * (uint32_t)sizeof(T) : BUF_OFF;
            const int ts = c * CHUNK_T + s_tq * GROUP_T;
            boff[s] = (ts < L && c < c_end) ? bc_row_off + (uint32_t)ts * (uint32_t)sizeof(T) : BUF_OFF;
        }
        ru_[0] = io8<T>::load_buf(bu, off[0]); ru_[1] = io8<T>::load_buf(bu, off[1]);
        if constexpr (FUSED_KS == 0) { rd_[0] = io8<T>::load_buf(bd, off[0]); rd_[1] = io8<T>::load_buf(bd, off[1]); }
        rz_[0] = io8<T>::load_buf(bz, off[0]); rz_[1] = io8<T>::load_buf(bz, off[1]);
        rp_[0] = io8<T>::load_buf(bp, off[0]); rp_[1] = io8<T>::load_buf(bp, off[1]);
        rbc_[0] = io4<T>::load_buf(bbc, boff[0]); rbc_[1] = io4<T>::load_buf(bbc, boff[1]);
      }
    };
    typename io8<T>::packed held_y{}, held_o{};
    if constexpr (FUSED_KS > 0) {
        issue_r(c_begin);
        stage_r();
        __syncthreads();
        project();
        __syncthreads();   // s_rT is rewritten in the first chunk's phase A
        issue_r(c_begin + 1);
    }
    uint32_t touched = 0u;
    if (BCFIX != 3 && !PAT) touched = touch(c_begin * CHUNK_T);

    // One chunk; the slot of its prefetched inputs (chunk index from c_begin, mod PF) is a compile-time
    // constant, so the prefetch registers are addressed statically and the loads just issued are
    // not touched again before their chunk comes up.
    auto do_chunk = [&](const int c, auto slot_tag) {
        constexpr int SLOT = decltype(slot_tag)::value;
        float u8[SLICE], z8[SLICE], v8[SLICE];
        const int tc = c * CHUNK_T;
        const int t0 = tc + pq * SLICE;
        const int nv = min(max(L - t0, 0), SLICE);
        // ---- A: pointwise pre-processing --------------------------------------------
        const typename io8<T>::raw ru = ru_[SLOT], rd = rd_[SLOT], rz = rz_[SLOT];
        const typename io4<T>::raw rbc = rbc_[SLOT];
        float p8[SLICE];
        if constexpr (VEC) {
            if (acc_on) io8<T>::unpack(rp_[SLOT], p8);   // uniform: only with more than 16 states
        }
        if constexpr (PAT) {
            float bc4[GROUP_T];
            io4<T>::unpack(rbc, bc4);
            *reinterpret_cast<float4*>(&s_bc[s_which][s_tq][s_n][0]) = make_float4(bc4[0], bc4[1], bc4[2], bc4[3]);
        }
        io8<T>::unpack(ru, u8);
        if constexpr (FUSED_KS > 0) {   // delta_raw of this chunk: left in s_raw by this same wave (project)
            const float4 d0v = *reinterpret_cast<const float4*>(&s_raw[pr][pq * SLICE]);
            const float4 d1v = *reinterpret_cast<const float4*>(&s_raw[pr][pq * SLICE + 4]);
            const float raw[SLICE] = {d0v.x, d0v.y, d0v.z, d0v.w, d1v.x, d1v.y, d1v.z, d1v.w};
#pragma unroll
            for (int j = 0; j < SLICE; ++j) v8[j] = bf16_to_f32(bf16_t(f32_to_bf16_bits(raw[j])));   // as the stored delta would be
        } else {
            io8<T>::unpack(rd, v8);
        }
        if (has_z) io8<T>::unpack(rz, z8);
        {
            float dt8[SLICE], du8[SLICE];
            // PAT without the in-kernel projection: a slice is whole or empty, and an empty one was read as
            // zeros; a bias of -1e30 (0 without softplus) then makes its step sizes exactly 0, the identity of
            // the recurrence, without a select per element
            constexpr bool ZERO_BY_BIAS = PAT && FUSED_KS == 0;
            const float bias_e = !ZERO_BY_BIAS || nv == SLICE ? bias : (softplus ? -1e30f : 0.0f);
#pragma unroll
            for (int j = 0; j < SLICE; ++j) {
                float x = v8[j] + bias_e, sp, sg;
                if (softplus) softplus_sigmoid(x, sp, sg); else sp = x;
                if constexpr (!ZERO_BY_BIAS) sp = (j < nv) ? sp : 0.0f;
                dt8[j] = sp;
                du8[j] = ZOH ? u8[j] : sp * u8[j];
                if (AGG) sum_dt += sp;
            }
            float4* pd4 = reinterpret_cast<float4*>(&s_dt[pr][pq * SLICE]);
            float4* pu4 = reinterpret_cast<float4*>(&s_du[pr][pq * SLICE]);
            pd4[0] = make_float4(dt8[0], dt8[1], dt8[2], dt8[3]);
            pd4[1] = make_float4(dt8[4], dt8[5], dt8[6], dt8[7]);
            pu4[0] = make_float4(du8[0], du8[1], du8[2], du8[3]);
            pu4[1] = make_float4(du8[4], du8[5], du8[6], du8[7]);
        }
        // The touch of the next chunk's B and C goes here, after the wait for this chunk's u,
        // delta and z: the value touched a chunk ago is older than those and costs no wait of
        // its own.
        if constexpr (!PAT) {
            consume_touch(touched);
            if (BCFIX != 3) touched = touch((c + 1) * CHUNK_T);
        }
        // checkpoint: the state entering every CKPT_T-step block (read back by the backward pass)
        auto save_ckpt = [&](int block) {
            if constexpr (AGG) return;
            if constexpr (VEC) {   // the block's 64 rows x 16 states; nothing is written if there is no block or no buffer
                const bool on = a.ckpt && block * CKPT_T < L;
                const rsrc_t bc = make_rsrc(a.ckpt + (((long)block * a.B + b) * a.D + d0) * NPAD,
                                            on ? (uint32_t)rows_here * NPAD * (uint32_t)sizeof(float) : 0u);
                buf_store16(bc, (uint32_t)(lane * NPAD + w * STATES_PER_LANE) * (uint32_t)sizeof(float),
                            make_uint4(__float_as_uint(h[0]), __float_as_uint(h[1]), __float_as_uint(h[2]), __float_as_uint(h[3])));
            } else if (a.ckpt && s_ok && block * CKPT_T < L) {
                float4* ck = reinterpret_cast<float4*>(a.ckpt + (((long)block * a.B + b) * a.D + sd) * NPAD) + w;
                *ck = make_float4(h[0], h[1], h[2], h[3]);
            }
        };
        save_ckpt(c * (CHUNK_T / CKPT_T));
        if constexpr (PAIR) {
            if constexpr (SLOT == 1) issue_pair(c + 1);
        } else {
            if (VEC || c + PF < c_end) issue_loads(c + PF, slot_tag);  // in flight during the scans below (VEC: switched off past the end, not branched around)
        }
        if constexpr (FUSED_KS > 0) {
            stage_r();          // r of chunk c + 1, requested a chunk ago; read by project() after the recurrence
            issue_r(c + 2);
        }
        __syncthreads();
        // ---- B: sequential recurrence over the chunk ---------------------------------
        __builtin_amdgcn_s_setprio(2);   // raised wave priority for the recurrence (see scan_bwd_kernel)
        constexpr int NG = CHUNK_T / GROUP_T;
        bc_group<T> Bg[2][STATES_PER_LANE], Cg[2][STATES_PER_LANE];
        constexpr int FB = 1;            // staged: groups fetched together (two gain nothing and spill scalar registers)
        bcs_group<T> Sg[2 * FB];
        const T* __restrict__ const sbc_chunk = STAGED ? sbc + (long)(tc / GROUP_T) * STAGE_GROUP : nullptr;
        auto fetch_bc = [&](int g, int slot) {
            if constexpr (PAT) {
                return;
            } else if constexpr (STAGED) {
                Sg[slot] = load_bcs<T>(sbc_chunk + g * STAGE_GROUP);
            } else {
#pragma unroll
                for (int k = 0; k < STATES_PER_LANE; ++k) {
                    if (!BFIX) Bg[slot][k] = load_bc<T, VEC, !FULLN>(gB[k], tc + g * GROUP_T, L, n_ok[k]);
                    if (!CFIX && !AGG) Cg[slot][k] = load_bc<T, VEC, !FULLN>(gC[k], tc + g * GROUP_T, L, n_ok[k]);
                }
            }
        };
        auto Bval = [&](int slot, int k, int j) -> float {
            if constexpr (STAGED) return Sg[slot].B(k, j); else return BFIX ? Bf[k] : Bg[slot][k].get(j);
        };
        auto Cval = [&](int slot, int k, int j) -> float {
            if constexpr (STAGED) return Sg[slot].C(k, j); else return CFIX ? Cf[k] : Cg[slot][k].get(j);
        };
        // Scalar loads return out of order and share their counter with LDS reads, so a wait
        // for either drains both: the step sizes of the whole chunk are read from LDS before
        // the loop, and inside it only the scalar loads of the next group are outstanding.
        float4 dtc[NG], duc[NG], Bpc[PAT ? NG : 1], Cpc[PAT ? NG : 1];
        const int pat = slot_state(w, lane & 3, a.il);   // PAT: the state of slot lane % 4
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            dtc[g] = *reinterpret_cast<const float4*>(&s_dt[lane][g * GROUP_T]);
            duc[g] = *reinterpret_cast<const float4*>(&s_du[lane][g * GROUP_T]);
            if constexpr (PAT) {
                Bpc[g] = *reinterpret_cast<const float4*>(&s_bc[0][g][pat][0]);
                if (!AGG) Cpc[g] = *reinterpret_cast<const float4*>(&s_bc[1][g][pat][0]);
            }
        }
        if constexpr (STAGED) {
#pragma unroll
            for (int i = 0; i < FB; ++i) fetch_bc(i, i);
        } else {
            fetch_bc(0, 0);
        }
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            const int cur = STAGED ? g % (2 * FB) : (g & 1);
            if constexpr (!STAGED) {
                if (g + 1 < NG) fetch_bc(g + 1, cur ^ 1);  // in flight while group g is consumed
            }
            const int tl = g * GROUP_T;  // step within the chunk
            const float4 dt4 = dtc[g], du4 = duc[g];
            if (g > 0 && tl % CKPT_T == 0) save_ckpt((tc + tl) / CKPT_T);
            float yp[GROUP_T];
#pragma unroll
            for (int j = 0; j < GROUP_T; ++j) {
                const float dt = f4_get(dt4, j), du = f4_get(du4, j);
                float y = 0.0f;
                if constexpr (CPLX) {
#pragma unroll
                    for (int k = 0; k < STATES_PER_LANE; k += 2) {
                        const cplx ab = complex_decay(dt, A2[k], An[k + 1]);         // Eq. 4 over C
                        const float br = du * Bval(cur, k, j);
                        const float bi = du * Bval(cur, k + 1, j);
                        const float hr = fmaf(ab.re, h[k], fmaf(-ab.im, h[k + 1], br));  // Eq. 2a over C
                        const float hi = fmaf(ab.im, h[k], fmaf(ab.re, h[k + 1], bi));
                        h[k] = hr;
                        h[k + 1] = hi;
                        if (!AGG) {                                                  // Re(C h)
                            y = fmaf(Cval(cur, k, j), hr, y);
                            y = fmaf(-Cval(cur, k + 1, j), hi, y);
                        }
                    }
                } else if constexpr (PAT) {
                    float bu[STATES_PER_LANE];
                    input_step_dpp<SPL>(bu, f4_get(Bpc[g], j), du);
#pragma unroll
                    for (int k = 0; k < SPL; ++k) {
                        const float x2 = dt * A2[k];
                        const float abar = exp2_fast(x2);                            // Eq. 4
                        if (ZOH) bu[k] *= zoh_phi_fast(dt, x2, abar, invA[k]);
                        h[k] = fmaf(abar, h[k], bu[k]);                              // Eq. 2a
                    }
                    if (!AGG) readout_step_dpp<SPL>(y, f4_get(Cpc[g], j), h);        // Eq. 2b
                } else {
#pragma unroll
                    for (int k = 0; k < SPL; ++k) {
                        const float abar = exp2_fast(dt * A2[k]);                    // Eq. 4
                        float bu = du * Bval(cur, k, j);
                        if (ZOH) bu *= zoh_phi(dt, An[k], invA[k], abar, false).phi;
                        h[k] = fmaf(abar, h[k], bu);                                 // Eq. 2a
                        if (!AGG) y = fmaf(Cval(cur, k, j), h[k], y);                         // Eq. 2b
                    }
                }
                yp[j] = y;
                if constexpr (STAGED) {
                    // The next group's load is issued after this group's first step, i.e. after
                    // the wait for this group's own operands, so that that wait does not drain
                    // it; the scheduling barriers keep the compiler from moving it either way.
                    if (j == 0 && g % FB == 0 && g + FB < NG) {
                        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                        for (int i = 0; i < FB; ++i) fetch_bc(g + FB + i, (g + FB + i) % (2 * FB));
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
            if (!AGG)
                *reinterpret_cast<float4*>(&s_yp[w][lane][tl]) = make_float4(yp[0], yp[1], yp[2], yp[3]);
        }
        // delta_raw of the next chunk, before the barrier: the next phase A rewrites s_rT after it
        if (c + 1 < c_end) project();
        __syncthreads();
        // ---- C: pointwise post-processing --------------------------------------------
        __builtin_amdgcn_s_setprio(0);
        if (!AGG) {
            float y8[SLICE];
#pragma unroll
            for (int j = 0; j < SLICE; ++j) y8[j] = has_D ? Dsk * u8[j] : 0.0f;
#pragma unroll
            for (int ww = 0; ww < NWAVES; ++ww) {
                const float4 p0 = *reinterpret_cast<const float4*>(&s_yp[ww][pr][pq * SLICE]);
                const float4 p1 = *reinterpret_cast<const float4*>(&s_yp[ww][pr][pq * SLICE + 4]);
                y8[0] += p0.x; y8[1] += p0.y; y8[2] += p0.z; y8[3] += p0.w;
                y8[4] += p1.x; y8[5] += p1.y; y8[6] += p1.z; y8[7] += p1.w;
            }
            const int nvs = p_ok ? nv : 0;
            if constexpr (VEC) {   // states beyond the first 16: add to what the earlier groups left
                if (acc_on) {
#pragma unroll
                    for (int j = 0; j < SLICE; ++j) y8[j] += p8[j];
                }
            } else if (a.acc_y) {
                const T* prev = (has_z ? static_cast<const T*>(a.ysave) : static_cast<const T*>(a.out)) + prow * L + t0;
                io8<T>::unpack(io8<T>::template load<VEC>(prev, nvs), p8);
#pragma unroll
                for (int j = 0; j < SLICE; ++j) y8[j] += p8[j];
            }
            const uint32_t off = nv == SLICE ? row_off + (uint32_t)t0 * (uint32_t)sizeof(T) : BUF_OFF;
            if constexpr (PAIR) {
                const typename io8<T>::packed py = io8<T>::pack(y8);   // y before the gate, for the backward pass's dz (if kept)
                if (has_z) {
#pragma unroll
                    for (int j = 0; j < SLICE; ++j) y8[j] *= z8[j] * sigmoid_fast(z8[j]);
                }
                const typename io8<T>::packed po = io8<T>::pack(y8);
                if (SLOT == 0 && c + 1 < c_end) {   // wait for the odd chunk
                    held_y = py;
                    held_o = po;
                } else {
                    // the even chunk before an odd one is whole; a lone even chunk has nothing waiting
                    const uint32_t off_e = SLOT == 1 ? row_off + (uint32_t)(t0 - CHUNK_T) * (uint32_t)sizeof(T) : BUF_OFF;
                    io8<T>::store_packed(by, off_e, held_y);
                    io8<T>::store_packed(by, off, py);
                    io8<T>::store_packed(bo, off_e, held_o);
                    io8<T>::store_packed(bo, off, po);
                }
            } else if constexpr (VEC) {
                io8<T>::store_buf(by, off, y8);   // y before the gate, for the backward pass's dz (if kept)
                if (has_z) {
#pragma unroll
                    for (int j = 0; j < SLICE; ++j) y8[j] *= z8[j] * sigmoid_fast(z8[j]);
                }
                io8<T>::store_buf(bo, off, y8);
            } else {
                if (has_z) {
                    if (a.ysave)  // y before the gate, for the backward pass's dz
                        io8<T>::template store<VEC>(static_cast<T*>(a.ysave) + prow * L + t0, y8, nvs);
#pragma unroll
                    for (int j = 0; j < SLICE; ++j) y8[j] *= z8[j] * sigmoid_fast(z8[j]);
                }
                io8<T>::template store<VEC>(gout + t0, y8, nvs);
            }
        }
        // no barrier needed here: the next phase A writes s_dt/s_du, which every wave has
        // finished reading (barrier above), and s_yp is rewritten only after the next barrier
    };
    for (int c = c_begin; c < c_end; c += PF) {
        do_chunk(c, std::integral_constant<int, 0>{});
        if constexpr (PF > 1) {
            if (c + 1 < c_end) do_chunk(c + 1, std::integral_constant<int, 1>{});
        }
    }

    if (AGG) {
        if (s_ok) {
            float4* dst = reinterpret_cast<float4*>(a.seg_h + ((long)seg * a.B * a.D + srow) * NPAD) + w;
            *dst = make_float4(h[0], h[1], h[2], h[3]);
        }
        sum_dt += __shfl_xor(sum_dt, 1);
        sum_dt += __shfl_xor(sum_dt, 2);
        if (p_ok && pq == 0) a.seg_sumdt[(long)seg * a.B * a.D + prow] = sum_dt;
    } else if (a.h_last && s_ok && seg == a.nseg - 1) {
#pragma unroll
        for (int k = 0; k < STATES_PER_LANE; ++k)
            if (n_ok[k]) a.h_last[srow * NS + slot_state(w, k, a.il)] = h[k];
    }
}

// Turns the segments' local end states into incoming states, in place:
// in[1] = loc[0];  in[s+1] = exp(A * sum_dt[s]) * in[s] + loc[s]   (one thread per (b,d,n)).
__global__ void carry_fwd_kernel(const FwdArgs a)
{
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const long rows = (long)a.B * a.D;
    if (i >= rows * NPAD) return;
    const long row = i / NPAD;
    const int n = position_state((int)(i % NPAD), a.il), d = row % a.D;   // the state this slot of the record holds
    const float A2 = n < a.N ? a.A[(long)d * a.NS + n] * LOG2E : 0.0f;
    // complex state: slots (n, n^1) are (re, im) of one state; the thread carries both parts
    // and writes its own (slot n even: real part)
    const bool cplx_state = a.flags & F_COMPLEX;
    const long ip = i ^ 1;
    const float A2r = cplx_state && (n & ~1) < a.N ? a.A[(long)d * a.NS + (n & ~1)] * LOG2E : 0.0f;
    const float Aim = cplx_state && (n | 1) < a.N ? a.A[(long)d * a.NS + (n | 1)] : 0.0f;
    float carry = a.seg_h[i];  // loc[0]: already includes h0
    float other = cplx_state ? a.seg_h[ip] : 0.0f;
    // Segments are taken CARRY_BATCH at a time: their loads do not depend on the carry, so
    // they are issued together and only the multiply-adds form the serial chain.
    constexpr int CARRY_BATCH = 16;
    for (int s0 = 1; s0 < a.nseg; s0 += CARRY_BATCH) {
        float loc[CARRY_BATCH], locp[CARRY_BATCH], sdt[CARRY_BATCH];
#pragma unroll
        for (int j = 0; j < CARRY_BATCH; ++j) {
            const int s = s0 + j;
            loc[j] = s < a.nseg - 1 ? a.seg_h[(long)s * rows * NPAD + i] : 0.0f;   // the last segment has no aggregate
            locp[j] = (cplx_state && s < a.nseg - 1) ? a.seg_h[(long)s * rows * NPAD + ip] : 0.0f;
            sdt[j] = s < a.nseg - 1 ? a.seg_sumdt[(long)s * rows + row] : 0.0f;
        }
#pragma unroll
        for (int j = 0; j < CARRY_BATCH; ++j) {
            const int s = s0 + j;
            if (s < a.nseg) {
                a.seg_h[(long)s * rows * NPAD + i] = carry;  // incoming state of segment s
                if (cplx_state) {
                    const cplx ab = complex_decay(sdt[j], A2r, Aim);
                    const float re = (n & 1) ? other : carry, im = (n & 1) ? carry : other;
                    const float nre = fmaf(ab.re, re, -ab.im * im) + ((n & 1) ? locp[j] : loc[j]);
                    const float nim = fmaf(ab.im, re, ab.re * im) + ((n & 1) ? loc[j] : locp[j]);
                    carry = (n & 1) ? nim : nre;
                    other = (n & 1) ? nre : nim;
                } else {
                    carry = fmaf(exp2_fast(A2 * sdt[j]), carry, loc[j]);
                }
            }
        }
    }
}

// Single-token step: 4 lanes per row, 4 states each; the state is read and written once,
// in place.  With N == 16 every per-state operand (state, A, B_t, C_t) is one aligned
// 16- or 8-byte access per lane.
template <typename T, bool FULLN, bool ZOH>
__global__ void __launch_bounds__(256) step_kernel(const StepArgs a)
{
    const long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const long rowi = gid >> 2;
    const int q = gid & 3;
    const long rows = (long)a.B * a.D;
    const bool row_ok = rowi < rows;
    const long row = row_ok ? rowi : rows - 1;
    const int b = row / a.D, d = row % a.D;
    const int N = a.N;

    const T* u_t = static_cast<const T*>(a.u_t);
    const T* dl_t = static_cast<const T*>(a.delta_t);
    const T* z_t = static_cast<const T*>(a.z_t);
    const T* B_t = static_cast<const T*>(a.B_t);
    const T* C_t = static_cast<const T*>(a.C_t);
    // time-invariant B / C are (D,N) float32 parameters; the launcher sends them down the generic path
    const bool bfix = !FULLN && (a.flags & F_B_FIXED), cfix = !FULLN && (a.flags & F_C_FIXED);
    auto ld = [](const T* p, long i) -> float {
        if constexpr (sizeof(T) == 2) return bf16_to_f32(p[i]); else return p[i];
    };
    // Every global load of the thread is requested here (and, on the vector path, right below),
    // back to back: optional operands through a valid stand-in pointer, and no arithmetic on a
    // loaded value in between, either of which would make the compiler wait for one load before
    // issuing the next -- four memory round trips instead of one.
    const bool has_bias = a.flags & F_HAS_DELTA_BIAS, has_D = a.flags & F_HAS_D, has_z = a.flags & F_HAS_Z;
    const T u_raw = u_t[row], dl_raw = dl_t[row], z_raw = (has_z ? z_t : u_t)[row];
    const float bias_raw = (has_bias ? a.bias : a.A)[has_bias ? d : 0];
    const float D_raw = (has_D ? a.Dskip : a.A)[has_D ? d : 0];
    float4 h4_first = make_float4(0.f, 0.f, 0.f, 0.f), A4_first = h4_first;
    uint4 B_first = make_uint4(0u, 0u, 0u, 0u), C_first = B_first;   // bf16: two words each; float: four
    if constexpr (FULLN) {
        h4_first = *reinterpret_cast<const float4*>(a.h + row * N + q * STATES_PER_LANE);
        A4_first = *reinterpret_cast<const float4*>(a.A + (long)d * NPAD + q * STATES_PER_LANE);
        const long bo = (long)b * a.bc_stride + q * STATES_PER_LANE;
        if constexpr (sizeof(T) == 2) {
            const uint2 Bw = *reinterpret_cast<const uint2*>(B_t + bo), Cw = *reinterpret_cast<const uint2*>(C_t + bo);
            B_first.x = Bw.x; B_first.y = Bw.y; C_first.x = Cw.x; C_first.y = Cw.y;
        } else {
            B_first = *reinterpret_cast<const uint4*>(B_t + bo);
            C_first = *reinterpret_cast<const uint4*>(C_t + bo);
        }
    }
    auto cvt = [](T v) -> float {
        if constexpr (sizeof(T) == 2) return bf16_to_f32(v); else return v;
    };
    const float u = cvt(u_raw);
    float x = cvt(dl_raw) + (has_bias ? bias_raw : 0.0f);
    float dt = x, sg;
    if (a.flags & F_DELTA_SOFTPLUS) softplus_sigmoid(x, dt, sg);
    const float du = ZOH ? u : dt * u, dt2 = dt * LOG2E;

    float y = 0.0f;
    // 16 states per pass: one pass when N <= 16 (always so on the vector path)
    for (int n0 = 0; n0 < (FULLN ? NPAD : N); n0 += NPAD) {
        float hv[STATES_PER_LANE], Av[STATES_PER_LANE], Bv[STATES_PER_LANE], Cv[STATES_PER_LANE];
        float* hp = a.h + row * N + n0 + q * STATES_PER_LANE;
        if (FULLN) {   // one pass; loaded above
            const float4 h4 = h4_first, A4 = A4_first;
            hv[0] = h4.x; hv[1] = h4.y; hv[2] = h4.z; hv[3] = h4.w;
            Av[0] = A4.x; Av[1] = A4.y; Av[2] = A4.z; Av[3] = A4.w;
            if constexpr (sizeof(T) == 2) {
                Bv[0] = bf16_lo(B_first.x); Bv[1] = bf16_hi(B_first.x); Bv[2] = bf16_lo(B_first.y); Bv[3] = bf16_hi(B_first.y);
                Cv[0] = bf16_lo(C_first.x); Cv[1] = bf16_hi(C_first.x); Cv[2] = bf16_lo(C_first.y); Cv[3] = bf16_hi(C_first.y);
            } else {
                Bv[0] = __uint_as_float(B_first.x); Bv[1] = __uint_as_float(B_first.y);
                Bv[2] = __uint_as_float(B_first.z); Bv[3] = __uint_as_float(B_first.w);
                Cv[0] = __uint_as_float(C_first.x); Cv[1] = __uint_as_float(C_first.y);
                Cv[2] = __uint_as_float(C_first.z); Cv[3] = __uint_as_float(C_first.w);
            }
        } else {
#pragma unroll
            for (int k = 0; k < STATES_PER_LANE; ++k) {
                const int n = n0 + q * STATES_PER_LANE + k;
                const bool ok = n < N;
                hv[k] = ok ? hp[k] : 0.0f;
                Av[k] = ok ? a.A[(long)d * N + n] : 0.0f;
                Bv[k] = !ok ? 0.0f : bfix ? static_cast<const float*>(a.B_t)[(long)d * N + n] : ld(B_t, (long)b * a.bc_stride + n);
                Cv[k] = !ok ? 0.0f : cfix ? static_cast<const float*>(a.C_t)[(long)d * N + n] : ld(C_t, (long)b * a.bc_stride + n);
            }
        }
        if (a.flags & F_COMPLEX) {   // slots (0,1) and (2,3) are (re, im) of two complex states
#pragma unroll
            for (int k = 0; k < STATES_PER_LANE; k += 2) {
                const cplx ab = complex_decay(dt, Av[k] * LOG2E, Av[k + 1]);
                const float hr = fmaf(ab.re, hv[k], fmaf(-ab.im, hv[k + 1], du * Bv[k]));
                const float hi = fmaf(ab.im, hv[k], fmaf(ab.re, hv[k + 1], du * Bv[k + 1]));
                hv[k] = hr;
                hv[k + 1] = hi;
                y = fmaf(Cv[k], hr, fmaf(-Cv[k + 1], hi, y));
            }
        } else {
#pragma unroll
            for (int k = 0; k < STATES_PER_LANE; ++k) {
                const float abar = exp2_fast(dt2 * Av[k]);                  // Eq. 4
                float bu = du * Bv[k];
                if (ZOH) bu *= zoh_phi(dt, Av[k], Av[k] != 0.0f ? 1.0f / Av[k] : 0.0f, abar, false).phi;
                hv[k] = fmaf(abar, hv[k], bu);                              // Eq. 2a
                y = fmaf(Cv[k], hv[k], y);                                  // Eq. 2b
            }
        }
        if (row_ok) {
            if (FULLN) {
                *reinterpret_cast<float4*>(hp) = make_float4(hv[0], hv[1], hv[2], hv[3]);
            } else {
#pragma unroll
                for (int k = 0; k < STATES_PER_LANE; ++k)
                    if (n0 + q * STATES_PER_LANE + k < N) hp[k] = hv[k];
            }
        }
    }
    // sum over the 4 lanes of the row
    y += __shfl_xor(y, 1);
    y += __shfl_xor(y, 2);
    if (has_D) y = fmaf(D_raw, u, y);
    if (has_z) {
        const float z = cvt(z_raw);
        y *= z * sigmoid_fast(z);
    }
    if (row_ok && q == 0) {
        if constexpr (sizeof(T) == 2) static_cast<bf16_t*>(a.out_t)[row] = bf16_t(f32_to_bf16_bits(y));
        else static_cast<float*>(a.out_t)[row] = y;
    }
}

// Single-token step, the common case at scale (N == 16, real state, first-order B-bar, selective
// B / C, vector-aligned operands): as step_kernel, with RPT batch entries (b, b + B/RPT, ...) of the
// same channel per thread.  A, bias and D are fetched once for them, and RPT state vectors per lane
// are in flight at once, which a streaming kernel this short needs to fill the memory pipeline.
template <typename T, int RPT>
__global__ void __launch_bounds__(256) step_multi_kernel(const StepArgs a)
{
    const long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const long rowi = gid >> 2;
    const int q = gid & 3;
    const int bpart = a.B / RPT;                       // the launcher checks B % RPT == 0
    const long rows_part = (long)bpart * a.D;
    const bool row_ok = rowi < rows_part;
    const long row0 = row_ok ? rowi : rows_part - 1;
    const int b0 = row0 / a.D, d = row0 % a.D;
    const T* u_t = static_cast<const T*>(a.u_t);
    const T* dl_t = static_cast<const T*>(a.delta_t);
    const T* z_t = static_cast<const T*>(a.z_t);
    const T* B_t = static_cast<const T*>(a.B_t);
    const T* C_t = static_cast<const T*>(a.C_t);
    const bool has_bias = a.flags & F_HAS_DELTA_BIAS, has_D = a.flags & F_HAS_D, has_z = a.flags & F_HAS_Z;
    // all loads first, none behind a branch or behind arithmetic on a loaded value (see step_kernel)
    float4 h4[RPT];
    T u_raw[RPT], dl_raw[RPT], z_raw[RPT];
    uint4 Bw[RPT], Cw[RPT];
    long row[RPT];
#pragma unroll
    for (int i = 0; i < RPT; ++i) {
        const int b = b0 + i * bpart;
        row[i] = (long)b * a.D + d;
        h4[i] = *reinterpret_cast<const float4*>(a.h + row[i] * NPAD + q * STATES_PER_LANE);
        u_raw[i] = u_t[row[i]];
        dl_raw[i] = dl_t[row[i]];
        z_raw[i] = (has_z ? z_t : u_t)[row[i]];
        const long bo = (long)b * a.bc_stride + q * STATES_PER_LANE;
        Bw[i] = make_uint4(0u, 0u, 0u, 0u);
        Cw[i] = Bw[i];
        if constexpr (sizeof(T) == 2) {
            const uint2 x = *reinterpret_cast<const uint2*>(B_t + bo), y = *reinterpret_cast<const uint2*>(C_t + bo);
            Bw[i].x = x.x; Bw[i].y = x.y; Cw[i].x = y.x; Cw[i].y = y.y;
        } else {
            Bw[i] = *reinterpret_cast<const uint4*>(B_t + bo);
            Cw[i] = *reinterpret_cast<const uint4*>(C_t + bo);
        }
    }
    const float4 A4 = *reinterpret_cast<const float4*>(a.A + (long)d * NPAD + q * STATES_PER_LANE);
    const float bias_raw = (has_bias ? a.bias : a.A)[has_bias ? d : 0];
    const float D_raw = (has_D ? a.Dskip : a.A)[has_D ? d : 0];
    auto cvt = [](T v) -> float {
        if constexpr (sizeof(T) == 2) return bf16_to_f32(v); else return v;
    };
    const float Av[STATES_PER_LANE] = {A4.x * LOG2E, A4.y * LOG2E, A4.z * LOG2E, A4.w * LOG2E};
#pragma unroll
    for (int i = 0; i < RPT; ++i) {
        const float u = cvt(u_raw[i]);
        float x = cvt(dl_raw[i]) + (has_bias ? bias_raw : 0.0f);
        float dt = x, sg;
        if (a.flags & F_DELTA_SOFTPLUS) softplus_sigmoid(x, dt, sg);
        const float du = dt * u;
        float hv[STATES_PER_LANE] = {h4[i].x, h4[i].y, h4[i].z, h4[i].w}, Bv[STATES_PER_LANE], Cv[STATES_PER_LANE];
        if constexpr (sizeof(T) == 2) {
            Bv[0] = bf16_lo(Bw[i].x); Bv[1] = bf16_hi(Bw[i].x); Bv[2] = bf16_lo(Bw[i].y); Bv[3] = bf16_hi(Bw[i].y);
            Cv[0] = bf16_lo(Cw[i].x); Cv[1] = bf16_hi(Cw[i].x); Cv[2] = bf16_lo(Cw[i].y); Cv[3] = bf16_hi(Cw[i].y);
        } else {
            Bv[0] = __uint_as_float(Bw[i].x); Bv[1] = __uint_as_float(Bw[i].y); Bv[2] = __uint_as_float(Bw[i].z); Bv[3] = __uint_as_float(Bw[i].w);
            Cv[0] = __uint_as_float(Cw[i].x); Cv[1] = __uint_as_float(Cw[i].y); Cv[2] = __uint_as_float(Cw[i].z); Cv[3] = __uint_as_float(Cw[i].w);
        }
        float y = 0.0f;
#pragma unroll
        for (int k = 0; k < STATES_PER_LANE; ++k) {
            const float abar = exp2_fast(dt * Av[k]);                       // Eq. 4
            hv[k] = fmaf(abar, hv[k], du * Bv[k]);                          // Eq. 2a
            y = fmaf(Cv[k], hv[k], y);                                      // Eq. 2b
        }
        if (row_ok)
            *reinterpret_cast<float4*>(a.h + row[i] * NPAD + q * STATES_PER_LANE) = make_float4(hv[0], hv[1], hv[2], hv[3]);
        y += __shfl_xor(y, 1);
        y += __shfl_xor(y, 2);
        if (has_D) y = fmaf(D_raw, u, y);
        if (has_z) {
            const float z = cvt(z_raw[i]);
            y *= z * sigmoid_fast(z);
        }
        if (row_ok && q == 0) {
            if constexpr (sizeof(T) == 2) static_cast<bf16_t*>(a.out_t)[row[i]] = bf16_t(f32_to_bf16_bits(y));
            else static_cast<float*>(a.out_t)[row[i]] = y;
        }
    }
}

// Single-token step of the layer's decode (bf16 I/O): as step_kernel, but delta_t, B_t and C_t come
// from the float32 output P = [r; B; C] of the projection (the sum of STEP_NPARTS partial results,
// rounded to bf16 as the layer stores it) and delta_t = W_dt r_t + bias is formed here.  A workgroup
// owns 64 channels and a tile of BT = 16 or 8 batch entries.  It stages the tile's rows of P in LDS;
// four of its eight waves then form the 16 x 64 block of W_dt r_t on the matrix cores (one 16 x 16
// tile per wave, rows past the tile shadowing its last one, W_dt rows straight from global memory)
// and leave softplus(. + bias) in LDS, once per (b, d) instead of once per quarter; after that a
// thread is (channel d, quarter q, half of the batch tile) as in step_kernel and walks its BT / 2
// batch entries.  The 8-entry tile needs fewer registers (two workgroups per CU instead of one) and
// gives twice the workgroups; the launcher picks the tile from the number of workgroups each gives.  The state, u and z of those entries are
// requested before anything else, so that their latency overlaps the projection.  Real, first-order,
// selective B / C only; R <= 256 and a multiple of 8, N <= 16.
constexpr int SP_MFMA_ROWS = 16;                  // rows of the MFMA tile: the largest batch tile
constexpr int SP_THREADS = 512;                   // 64 channels x 4 quarters x 2 halves of the batch tile
constexpr int STEP_MAX_LDP = 256 + 2 * NPAD;      // R <= 256 and N <= 16 on this path
constexpr int SP_MAX_KSTEPS = 256 / 32;             // contraction steps of the delta projection (R <= 256)
constexpr int SP_LDP = STEP_MAX_LDP + 4;          // row stride of the staged P in floats: 16-byte rows, off the banks

template <bool FULLN, int SP_BT>
__global__ void __launch_bounds__(SP_THREADS) step_proj_kernel(const StepArgs a)
{
    static_assert(SP_BT == 8 || SP_BT == SP_MFMA_ROWS, "batch tile");
    constexpr int SP_PER = SP_BT / 2;                // batch entries per thread
    __shared__ __attribute__((aligned(16))) float s_p[SP_BT][SP_LDP];
    __shared__ float s_dt[SP_MFMA_ROWS][64];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int q = tid & 3, dl = (tid >> 2) & 63, half = tid >> 8;
    const int d0 = blockIdx.x * 64;
    const bool d_ok = d0 + dl < a.D;
    const int d = d_ok ? d0 + dl : a.D - 1;
    const int N = a.N, R = a.R;
    const int b0 = blockIdx.y * SP_BT;
    const int nbt = min(SP_BT, a.B - b0);            // batch entries of this tile
    const bf16_t* u_t = static_cast<const bf16_t*>(a.u_t);
    const bf16_t* z_t = static_cast<const bf16_t*>(a.z_t);
    auto as_stored = [](float v) -> float { return bf16_to_f32(bf16_t(f32_to_bf16_bits(v))); };

    // Everything the thread needs from global memory is requested here, in straight-line code
    // with no branch between the loads (optional operands are read through a valid stand-in
    // pointer and discarded) and no arithmetic on a loaded value: either would make the compiler
    // wait for that load before issuing the next, one memory latency after another.
    const int sq = q * STATES_PER_LANE;               // this quarter's first state
    const bool has_z = a.flags & F_HAS_Z, has_D = a.flags & F_HAS_D, has_bias = a.flags & F_HAS_DELTA_BIAS;
    const bf16_t* zp = has_z ? z_t : u_t;
    float hv[SP_PER][STATES_PER_LANE];
    bf16_t ub_raw[SP_PER], zb_raw[SP_PER];
#pragma unroll
    for (int i = 0; i < SP_PER; ++i) {
        const int b = min(b0 + half * SP_PER + i, a.B - 1);
        const long row = (long)b * a.D + d;
        if constexpr (FULLN) {
            const float4 h4 = *reinterpret_cast<const float4*>(a.h + row * N + sq);
            hv[i][0] = h4.x; hv[i][1] = h4.y; hv[i][2] = h4.z; hv[i][3] = h4.w;
        } else {
#pragma unroll
            for (int k = 0; k < STATES_PER_LANE; ++k) hv[i][k] = a.h[row * N + min(sq + k, N - 1)];   // a valid element; masked below
        }
        ub_raw[i] = u_t[row];
        zb_raw[i] = zp[row];
    }
    float A_raw[STATES_PER_LANE];
#pragma unroll
    for (int k = 0; k < STATES_PER_LANE; ++k) A_raw[k] = a.A[(long)d * N + min(sq + k, N - 1)];
    const float D_raw = (has_D ? a.Dskip : a.A)[has_D ? d : 0];

    // Waves 0-3 form the tile (batch entries) x (channels d0 + 16 * wave ..+15) of r W_dt^T after
    // the staging below.  Operand layout of the 16x16x32 bf16 MFMA: lane l holds row (column)
    // l % 16 of the first (second) operand at contraction indices 8 * (l / 16) ..+7; accumulator
    // element i of lane l is row 4 * (l / 16) + i, column l % 16.  Their pieces of W_dt are
    // requested now, with everything else (from a clamped, valid address; zeroed below where the
    // piece lies past R).
    const int dcol = 16 * (wave & 3) + (lane & 15);
    const int wrow = min(d0 + dcol, a.D - 1);
    const int ksub = 8 * (lane >> 4);
    union WFrag { unsigned short s[8]; bf16x8_t v; } wfrag[SP_MAX_KSTEPS];
    const float bias_raw = (has_bias ? a.bias : a.A)[has_bias ? wrow : 0];
    {
        const bf16_t* wp = static_cast<const bf16_t*>(a.W_dt) + (long)wrow * R;
#pragma unroll
        for (int i = 0; i < SP_MAX_KSTEPS; ++i)
            wfrag[i].v = *reinterpret_cast<const bf16x8_t*>(wp + min(32 * i + ksub, R - 8));   // R is a multiple of 8
    }

    {
        // P of the tile: all loads first (STEP_NPARTS x STAGE_ITEMS per thread, independent), then
        // the parts added in a fixed order and rounded as stored
        constexpr int STAGE_ITEMS = (SP_BT * STEP_MAX_LDP + SP_THREADS - 1) / SP_THREADS;
        const long part = (long)a.B * a.ldp;   // floats between partial results
        const int count = nbt * a.ldp;
        float v[STAGE_ITEMS][STEP_NPARTS];
#pragma unroll
        for (int j = 0; j < STAGE_ITEMS; ++j) {
            const int i = tid + SP_THREADS * j;
            const long g = (long)b0 * a.ldp + min(i, count - 1);
#pragma unroll
            for (int k = 0; k < STEP_NPARTS; ++k) v[j][k] = a.P[k * part + g];
        }
#pragma unroll
        for (int j = 0; j < STAGE_ITEMS; ++j) {
            const int i = tid + SP_THREADS * j;
            float s = v[j][0];
#pragma unroll
            for (int k = 1; k < STEP_NPARTS; ++k) s += v[j][k];
            if (i < count) s_p[i / a.ldp][i % a.ldp] = as_stored(s);
        }
    }
    __syncthreads();

    if (wave < 4) {
        const int arow = min(lane & 15, nbt - 1);             // rows past the end shadow the last one
        const float* pp = &s_p[arow][ksub];
        f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < SP_MAX_KSTEPS; ++i) {
            const int k = 32 * i;
            if (k < R) {                                      // uniform
                union { unsigned short s[8]; bf16x8_t v; } av;
#pragma unroll
                for (int e = 0; e < 8; ++e) av.s[e] = 0;
                if (k + ksub < R) {                           // R is a multiple of 8
                    const float4 p0 = *reinterpret_cast<const float4*>(pp + k);
                    const float4 p1 = *reinterpret_cast<const float4*>(pp + k + 4);
                    const float pv[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
#pragma unroll
                    for (int e = 0; e < 8; ++e) av.s[e] = (unsigned short)(__float_as_uint(pv[e]) >> 16);   // exact: rounded above
                }
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av.v, wfrag[i].v, acc, 0, 0, 0);
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float x = as_stored(acc[i]) + (has_bias ? bias_raw : 0.0f), dt = x, sg;
            if (a.flags & F_DELTA_SOFTPLUS) softplus_sigmoid(x, dt, sg);
            s_dt[4 * (lane >> 4) + i][dcol] = dt;
        }
    }
    __syncthreads();

    float Av[STATES_PER_LANE];
#pragma unroll
    for (int k = 0; k < STATES_PER_LANE; ++k) Av[k] = (sq + k < N) ? A_raw[k] * LOG2E : 0.0f;
    const float Dsk = has_D ? D_raw : 0.0f;
#pragma unroll
    for (int i = 0; i < SP_PER; ++i) {
        const int bl = half * SP_PER + i;
        if (bl >= nbt) break;
        if constexpr (!FULLN) {
#pragma unroll
            for (int k = 0; k < STATES_PER_LANE; ++k) hv[i][k] = (sq + k < N) ? hv[i][k] : 0.0f;
        }
        const long row = (long)(b0 + bl) * a.D + d;
        const float* pb = s_p[bl];
        const float dt = s_dt[bl][dl];
        const float u = bf16_to_f32(ub_raw[i]);
        const float du = dt * u;
        float Bq[STATES_PER_LANE], Cq[STATES_PER_LANE];
        if constexpr (FULLN) {
            const float4 b4 = *reinterpret_cast<const float4*>(pb + R + sq);
            const float4 c4 = *reinterpret_cast<const float4*>(pb + R + NPAD + sq);
            Bq[0] = b4.x; Bq[1] = b4.y; Bq[2] = b4.z; Bq[3] = b4.w;
            Cq[0] = c4.x; Cq[1] = c4.y; Cq[2] = c4.z; Cq[3] = c4.w;
        } else {
#pragma unroll
            for (int k = 0; k < STATES_PER_LANE; ++k) {
                const bool ok = sq + k < N;
                Bq[k] = ok ? pb[R + sq + k] : 0.0f;
                Cq[k] = ok ? pb[R + N + sq + k] : 0.0f;
            }
        }
        float y = 0.0f;
#pragma unroll
        for (int k = 0; k < STATES_PER_LANE; ++k) {
            const float abar = exp2_fast(dt * Av[k]);          // Eq. 4
            hv[i][k] = fmaf(abar, hv[i][k], du * Bq[k]);       // Eq. 2a
            y = fmaf(Cq[k], hv[i][k], y);                      // Eq. 2b
        }
        if (d_ok) {
            float* hp = a.h + row * N + sq;
            if constexpr (FULLN) {
                *reinterpret_cast<float4*>(hp) = make_float4(hv[i][0], hv[i][1], hv[i][2], hv[i][3]);
            } else {
#pragma unroll
                for (int k = 0; k < STATES_PER_LANE; ++k)
                    if (sq + k < N) hp[k] = hv[i][k];
            }
        }
        y += __shfl_xor(y, 1);
        y += __shfl_xor(y, 2);
        y = fmaf(Dsk, u, y);
        if (has_z) {
            const float z = bf16_to_f32(zb_raw[i]);
            y *= z * sigmoid_fast(z);
        }
        if (d_ok && q == 0) static_cast<bf16_t*>(a.out_t)[row] = bf16_t(f32_to_bf16_bits(y));
    }
}

// h_last for an empty sequence: h0 or zero
__global__ void copy_state_kernel(const float* __restrict__ src, float* __restrict__ dst, long n)
{
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src ? src[i] : 0.0f;
}

// Wave-packed copy of the selective B and C for the forward kernels (layout: FwdArgs::bcs).
// A thread writes the four steps of one (batch entry, state, group of steps, B or C).
// deal: a last group of fewer than 16 states is dealt out to the waves in turn (FwdArgs::il).
template <typename T>
__global__ void stage_bc_kernel(const T* __restrict__ Bm, const T* __restrict__ Cm, long bstride, T* __restrict__ dst,
                                int B, int NS, int L, int Lp, int deal)
{
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const int tgroups = Lp / GROUP_T, sgroups = (NS + NPAD - 1) / NPAD * NWAVES;   // every wave of every pass has a piece
    if (i >= (long)B * sgroups * tgroups * 2 * STATES_PER_LANE) return;
    const int r = (int)(i % (2 * STATES_PER_LANE));            // which * 4 + k
    const long piece = i / (2 * STATES_PER_LANE);
    const int tg = (int)(piece % tgroups);
    const int sg = (int)((piece / tgroups) % sgroups);
    const int b = (int)(piece / ((long)tgroups * sgroups));
    const int grp = sg / NWAVES;
    const int n = grp * NPAD + slot_state(sg % NWAVES, r % STATES_PER_LANE, deal && NS - grp * NPAD < NPAD), t = tg * GROUP_T;
    const T* src = (r >= STATES_PER_LANE ? Cm : Bm) + (long)b * bstride + (long)n * L + t;
    T v[GROUP_T];
#pragma unroll
    for (int j = 0; j < GROUP_T; ++j) v[j] = (n < NS && t + j < L) ? src[j] : T(0);
    T* out = dst + i * GROUP_T;
    if constexpr (sizeof(T) == 2) {
        *reinterpret_cast<uint2*>(out) = make_uint2(uint32_t(v[0]) | (uint32_t(v[1]) << 16), uint32_t(v[2]) | (uint32_t(v[3]) << 16));
    } else {
        *reinterpret_cast<float4*>(out) = make_float4(v[0], v[1], v[2], v[3]);
    }
}

int launch_stage_bc(const FwdArgs& a, void* bcs, int io_dtype, hipStream_t stream)
{
    // a carries all NS states here; whether a partial last group is dealt out depends on the path alone
    const int deal = a.vec_ok && !(a.flags & (F_EXACT_ZOH_B | F_B_FIXED | F_C_FIXED | F_COMPLEX));
    const long n = (long)a.B * ((a.NS + NPAD - 1) / NPAD * NWAVES) * (a.Lp / GROUP_T) * 2 * STATES_PER_LANE;
    const dim3 grid((unsigned)((n + 255) / 256));
    if (io_dtype == 0)
        stage_bc_kernel<float><<<grid, dim3(256), 0, stream>>>(static_cast<const float*>(a.Bm), static_cast<const float*>(a.Cm),
                                                               a.bc_bstride, static_cast<float*>(bcs), a.B, a.NS, a.L, a.Lp, deal);
    else
        stage_bc_kernel<bf16_t><<<grid, dim3(256), 0, stream>>>(static_cast<const bf16_t*>(a.Bm), static_cast<const bf16_t*>(a.Cm),
                                                                a.bc_bstride, static_cast<bf16_t*>(bcs), a.B, a.NS, a.L, a.Lp, deal);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

template <typename T, bool VEC, bool FULLN, bool ZOH, int BCFIX>
static void launch_fwd_fixed(const FwdArgs& a, hipStream_t stream)
{
    const int groups = (a.D + ROWS - 1) / ROWS;
    scan_fwd_kernel<T, VEC, FULLN, false, ZOH, BCFIX><<<dim3((unsigned)(a.B * groups), 1u), dim3(THREADS), 0, stream>>>(a);
}

// complex state: first-order B-bar only; selective or time-invariant B / C
template <typename T, bool VEC, bool FULLN, int BCFIX>
static void launch_fwd_complex(const FwdArgs& a, hipStream_t stream)
{
    const int groups = (a.D + ROWS - 1) / ROWS;
    const dim3 block(THREADS);
    if (a.nseg > 1) {
        scan_fwd_kernel<T, VEC, FULLN, true, false, BCFIX, true><<<dim3((unsigned)(a.B * groups), (unsigned)(a.nseg - 1)), block, 0, stream>>>(a);
        const long n = (long)a.B * a.D * NPAD;
        carry_fwd_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream>>>(a);
    }
    scan_fwd_kernel<T, VEC, FULLN, false, false, BCFIX, true><<<dim3((unsigned)(a.B * groups), (unsigned)a.nseg), block, 0, stream>>>(a);
}

// real state, selective B and C
template <typename T, bool VEC, bool FULLN, bool ZOH, int SPL>
static void launch_fwd_selective(const FwdArgs& a, hipStream_t stream)
{
    const int groups = (a.D + ROWS - 1) / ROWS;
    const dim3 block(THREADS);
    constexpr bool PAT = VEC;          // B and C through the LDS tile; otherwise the scalar path (repacked copy if there is one)
    if (a.nseg > 1) {
        if (PAT || a.bcs)
            scan_fwd_kernel<T, VEC, FULLN, true, ZOH, 0, false, !PAT, 0, SPL, PAT><<<dim3((unsigned)(a.B * groups), (unsigned)(a.nseg - 1)), block, 0, stream>>>(a);
        else
            scan_fwd_kernel<T, VEC, FULLN, true, ZOH, 0, false, false, 0, SPL, false><<<dim3((unsigned)(a.B * groups), (unsigned)(a.nseg - 1)), block, 0, stream>>>(a);
        const long n = (long)a.B * a.D * NPAD;
        carry_fwd_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream>>>(a);
    }
    if constexpr (sizeof(T) == 2 && VEC && !ZOH && SPL == STATES_PER_LANE) {
        if (a.W_dt) {   // the caller has checked: unsplit, R <= 256
            if (a.Rp <= 128)
                scan_fwd_kernel<T, VEC, FULLN, false, ZOH, 0, false, false, 4, SPL, true><<<dim3((unsigned)(a.B * groups), 1u), block, 0, stream>>>(a);
            else
                scan_fwd_kernel<T, VEC, FULLN, false, ZOH, 0, false, false, 8, SPL, true><<<dim3((unsigned)(a.B * groups), 1u), block, 0, stream>>>(a);
            return;
        }
    }
    if (PAT || a.bcs)
        scan_fwd_kernel<T, VEC, FULLN, false, ZOH, 0, false, !PAT, 0, SPL, PAT><<<dim3((unsigned)(a.B * groups), (unsigned)a.nseg), block, 0, stream>>>(a);
    else
        scan_fwd_kernel<T, VEC, FULLN, false, ZOH, 0, false, false, 0, SPL, false><<<dim3((unsigned)(a.B * groups), (unsigned)a.nseg), block, 0, stream>>>(a);
}

template <typename T, bool VEC, bool FULLN, bool ZOH>
static void launch_fwd_t(const FwdArgs& a, hipStream_t stream)
{
    const int groups = (a.D + ROWS - 1) / ROWS;
    const dim3 block(THREADS);
    // time-invariant B and/or C: never split (the planner keeps nseg == 1 for them)
    const int bcfix = ((a.flags & F_B_FIXED) ? 1 : 0) | ((a.flags & F_C_FIXED) ? 2 : 0);
    if constexpr (!ZOH) {
        if (a.flags & F_COMPLEX) {
            if (bcfix == 0) return launch_fwd_complex<T, VEC, FULLN, 0>(a, stream);
            if (bcfix == 1) return launch_fwd_complex<T, VEC, FULLN, 1>(a, stream);
            if (bcfix == 2) return launch_fwd_complex<T, VEC, FULLN, 2>(a, stream);
            return launch_fwd_complex<T, VEC, FULLN, 3>(a, stream);
        }
    }
    if (bcfix == 1) return launch_fwd_fixed<T, VEC, FULLN, ZOH, 1>(a, stream);
    if (bcfix == 2) return launch_fwd_fixed<T, VEC, FULLN, ZOH, 2>(a, stream);
    if (bcfix == 3) return launch_fwd_fixed<T, VEC, FULLN, ZOH, 3>(a, stream);
    if constexpr (VEC && !FULLN && !ZOH) {   // fewer than 16 states dealt out to the waves: kernels built for 1 or 2 slots per lane
        const int spl = slots_for(a.N, a.il);
        if (spl == 1) return launch_fwd_selective<T, VEC, FULLN, ZOH, 1>(a, stream);
        if (spl == 2) return launch_fwd_selective<T, VEC, FULLN, ZOH, 2>(a, stream);
    }
    launch_fwd_selective<T, VEC, FULLN, ZOH, STATES_PER_LANE>(a, stream);
}

int launch_fwd(const FwdArgs& a, int io_dtype, hipStream_t stream)
{
    if (a.L == 0) {
        if (a.h_last) {
            const long n = (long)a.B * a.D * a.NS;
            copy_state_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream>>>(
                (a.flags & F_HAS_H0) ? a.h0 : nullptr, a.h_last, n);
        }
        return hipGetLastError() == hipSuccess ? 0 : -1;
    }
    const bool fulln = a.N == NPAD;
    if (a.flags & F_EXACT_ZOH_B) {  // the variant is built for the fastest and the most general shape only
        if (io_dtype == 0) {
            if (a.vec_ok && fulln) launch_fwd_t<float, true, true, true>(a, stream);
            else launch_fwd_t<float, false, false, true>(a, stream);
        } else {
            if (a.vec_ok && fulln) launch_fwd_t<bf16_t, true, true, true>(a, stream);
            else launch_fwd_t<bf16_t, false, false, true>(a, stream);
        }
    } else if (io_dtype == 0) {
        if (a.vec_ok && fulln) launch_fwd_t<float, true, true, false>(a, stream);
        else if (a.vec_ok) launch_fwd_t<float, true, false, false>(a, stream);
        else launch_fwd_t<float, false, false, false>(a, stream);
    } else {
        if (a.vec_ok && fulln) launch_fwd_t<bf16_t, true, true, false>(a, stream);
        else if (a.vec_ok) launch_fwd_t<bf16_t, true, false, false>(a, stream);
        else launch_fwd_t<bf16_t, false, false, false>(a, stream);
    }
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

int launch_step(const StepArgs& a, int io_dtype, hipStream_t stream)
{
    const long lanes = (long)a.B * a.D * 4;
    const dim3 grid((unsigned)((lanes + 255) / 256)), block(256);
    // the vector path also needs B_t / C_t rows aligned to 8 (bf16) or 16 (float) bytes,
    // which N == 16 and the element-aligned base pointers checked by the caller give only
    // when the bases themselves are that aligned
    const size_t va = io_dtype == 0 ? 16 : 8;
    const bool vec = a.N == NPAD && !(a.flags & (F_B_FIXED | F_C_FIXED)) && (a.bc_stride * (io_dtype == 0 ? 4 : 2)) % va == 0 &&
                     reinterpret_cast<uintptr_t>(a.B_t) % va == 0 &&
                     reinterpret_cast<uintptr_t>(a.C_t) % va == 0 && reinterpret_cast<uintptr_t>(a.A) % 16 == 0;
    const bool zoh = a.flags & F_EXACT_ZOH_B;
    // Several batch entries per thread once that still leaves every CU its 2048 threads
    if (vec && !zoh && !(a.flags & F_COMPLEX)) {
        const long full = 256L * 2048;
        const int rpt = (a.B % 4 == 0 && lanes / 4 >= full) ? 4 : (a.B % 2 == 0 && lanes / 2 >= full) ? 2 : 1;
        if (rpt > 1) {
            const dim3 g((unsigned)((lanes / rpt + 255) / 256));
            if (io_dtype == 0) {
                if (rpt == 4) step_multi_kernel<float, 4><<<g, block, 0, stream>>>(a);
                else step_multi_kernel<float, 2><<<g, block, 0, stream>>>(a);
            } else {
                if (rpt == 4) step_multi_kernel<bf16_t, 4><<<g, block, 0, stream>>>(a);
                else step_multi_kernel<bf16_t, 2><<<g, block, 0, stream>>>(a);
            }
            return hipGetLastError() == hipSuccess ? 0 : -1;
        }
    }
#define SS_LAUNCH_STEP(T, V, Z) step_kernel<T, V, Z><<<grid, block, 0, stream>>>(a)
    if (io_dtype == 0) {
        if (vec) { if (zoh) SS_LAUNCH_STEP(float, true, true); else SS_LAUNCH_STEP(float, true, false); }
        else { if (zoh) SS_LAUNCH_STEP(float, false, true); else SS_LAUNCH_STEP(float, false, false); }
    } else {
        if (vec) { if (zoh) SS_LAUNCH_STEP(bf16_t, true, true); else SS_LAUNCH_STEP(bf16_t, true, false); }
        else { if (zoh) SS_LAUNCH_STEP(bf16_t, false, true); else SS_LAUNCH_STEP(bf16_t, false, false); }
    }
#undef SS_LAUNCH_STEP
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

int launch_step_projected(const StepArgs& a, hipStream_t stream)
{
    // One workgroup per CU is the fastest arrangement (the state streams while the projection's
    // dependent steps run), so: 8-entry batch tiles while they fit the chip's 256 CUs once, 16-entry
    // tiles while those still do, and 8-entry tiles again beyond that, where two of them share a CU
    // (measured at D = 2048, 4096, 5120 and batch 32 ... 256: the better tile by 5-15 % in every case).
    const long groups = (a.D + 63) / 64;
    const long n16 = groups * ((a.B + SP_MFMA_ROWS - 1) / SP_MFMA_ROWS), n8 = groups * ((a.B + 7) / 8);
    const bool wide = n8 > 256 && n16 <= 256;
    const dim3 grid((unsigned)groups, (unsigned)(wide ? (a.B + SP_MFMA_ROWS - 1) / SP_MFMA_ROWS : (a.B + 7) / 8));
    const dim3 block(SP_THREADS);
    if (a.N == NPAD) {
        if (wide) step_proj_kernel<true, SP_MFMA_ROWS><<<grid, block, 0, stream>>>(a);
        else step_proj_kernel<true, 8><<<grid, block, 0, stream>>>(a);
    } else {
        if (wide) step_proj_kernel<false, SP_MFMA_ROWS><<<grid, block, 0, stream>>>(a);
        else step_proj_kernel<false, 8><<<grid, block, 0, stream>>>(a);
    }
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // namespace ss
