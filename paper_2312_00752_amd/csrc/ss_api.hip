// C-ABI entry points: host-side validation and dispatch only (see include/ss_scan.h).
#include <hip/hip_runtime.h>

#include <atomic>

#include "ss_kernels.h"
#include "ss_layer.h"
#include "ss_scan.h"

// Scratch of ss_scan_fwd_static: lives in the library's device image, one copy per GPU.  In host
// code this name is only a handle for hipGetSymbolAddress; the device address it yields is what
// every kernel argument below uses.
static __device__ __align__(256) unsigned char scratch[SS_STATIC_SCRATCH_BYTES];

namespace {

constexpr uint32_t kFwdFlags = SS_DELTA_SOFTPLUS | SS_HAS_DELTA_BIAS | SS_HAS_D | SS_HAS_Z |
                               SS_HAS_H0 | SS_WRITE_H_LAST | SS_SAVE_FOR_BWD | SS_EXACT_ZOH_B |
                               SS_B_FIXED | SS_C_FIXED | SS_COMPLEX_STATE;
constexpr uint32_t kStepFlags = SS_DELTA_SOFTPLUS | SS_HAS_DELTA_BIAS | SS_HAS_D | SS_HAS_Z | SS_EXACT_ZOH_B |
                                SS_B_FIXED | SS_C_FIXED | SS_COMPLEX_STATE;

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
// Real numbers per state vector: a complex state is a (re, im) pair of slots, and everything
// below the validation works on slots.
inline int slots(const ss_fwd_params* p) { return p->dstate * ((p->flags & SS_COMPLEX_STATE) ? 2 : 1); }
inline int slots(const ss_step_params* p) { return p->dstate * ((p->flags & SS_COMPLEX_STATE) ? 2 : 1); }

// Split of the sequence across workgroups.  The scan kernels run one workgroup per 64 rows
// of a batch entry; when that fills the chip badly and the sequence is long, L is cut into
// segments (multiples of 64 steps) that are scanned
// concurrently and stitched with a carry pass (Appendix D: the scan continues from the
// state the previous chunk ended in; here the chunks run in parallel from aggregates).
struct SegPlan {
    int nseg, seg_len;
};
// Modelled duration (in steps of one unsplit workgroup running alone on its compute unit) of a
// launch of n equal workgroups of len steps each.  Two workgroups fit a compute unit and then
// each runs at about 3/4 of the speed it has alone (measured: 256 workgroups of 2048 steps
// take 1.01 ms, 512 take 1.35 ms), so the chip takes workgroups in rounds of 512.  A workgroup's
// set-up, pipeline fill and final stores cost about as much as 32 more steps (fitted to sweeps of
// the segment count at 160 x 16384, 192 x 2048 and 4 x 2^20 workgroups x steps).
double launch_cost(long n, long len)
{
    const double pair = 1.0 / 0.75, fixed = 32.0;
    const long full = n / 512, rest = n % 512;
    return ((double)len + fixed) * ((double)full * pair + (rest == 0 ? 0.0 : (rest <= 256 ? 1.0 : pair)));
}

long segment_length(int L, long nseg)
{
    // whole pairs of 32-step chunks: the forward kernel issues the traffic of an even chunk and the
    // odd one after it together
    long len = ((L + nseg - 1) / nseg + 63) / 64 * 64;
    // A segment length that is a large power of two makes every workgroup walk the memory
    // channels in lockstep (all segment starts alias); an odd multiple of 64 steps staggers them
    // (measured: 7-12 % on the 2^20-step workload).  Short segments are staggered only when
    // there are hundreds of them; otherwise the shorter last segment costs more than the
    // aliasing does (measured on 8K- and 64K-step sequences).
    if (nseg > 1 && len % 256 == 0) len += len >= 2048 ? 192 : (nseg >= 256 ? 64 : 0);
    return len;
}

SegPlan plan_segments(int B, int D, int L, uint32_t flags)
{
    const long wgs = (long)B * ((D + 63) / 64);
    SegPlan s{1, (L + 31) / 32 * 32};
    if (s.seg_len == 0) s.seg_len = 32;
    if (flags & (SS_B_FIXED | SS_C_FIXED)) return s;   // the time-invariant variants are not split
    if (L < 128) return s;
    // Pick the number of segments that the model says finishes first: the main pass over
    // wgs * nseg workgroups plus the aggregate pass over wgs * (nseg - 1) of them, which costs
    // about 0.36 of a main pass per step (measured over forward + backward).  Segments stay
    // at least 64 steps long (two forward chunks), and a launch within 8192 workgroups, which
    // bounds the aggregates' workspace.
    double best = launch_cost(wgs, s.seg_len);
    long best_n = 1;
    const long fit = 8192 / wgs > 2 ? 8192 / wgs : 2;
    const long longest = L / 64 < 4096 ? L / 64 : 4096;
    const long most = longest < fit ? longest : fit;
    for (long want = 2; want <= most; ++want) {
        const long len = segment_length(L, want);
        const long n = (L + len - 1) / len;   // what that length really gives
        if (n < 2) continue;
        const double c = launch_cost(wgs * n, len) + 0.36 * launch_cost(wgs * (n - 1), len);
        if (c < best * 0.97) { best = c; best_n = want; }   // more segments only for a clear gain
    }
    if (best_n > 1) {
        s.seg_len = (int)segment_length(L, best_n);
        s.nseg = (L + s.seg_len - 1) / s.seg_len;
    }
    return s;
}

// Workspace layouts, each block 256-byte aligned.
//   forward only:  [io pre-gate y B*D*L, only with a gate and more than 16 states]
//                  [float seg_h nseg*B*D*16][float seg_sumdt nseg*B*D]        (only when split)
//   with backward: [float checkpoints groups*nck*B*D*16][io pre-gate y B*D*L, only with a gate]
//                  [seg_h][seg_sumdt][float seg_g nseg*B*D*16]                 (only when split)
//                  [float dA partials nseg*B*D*16][float dD partials nseg*B*D][float dbias partials nseg*B*D]
//                  [float dB partials B*D*16][float dC partials B*D*16]    (only for a time-invariant B / C)
//   both end with: [io staged B and C, B * ceil16(slots) * Lp * 2]    (only for a real state with selective B and C)
// where Lp is L rounded up to a whole 32-step chunk.
struct WsLayout {
    size_t ckpt_off, ckpt_group, y_off, segh_off, segdt_off, segg_off, dA_off, dD_off, db_off, dBf_off, dCf_off;
    size_t bcs_off, total;
    int Lp;
    SegPlan plan;
};
// The forward kernels read a real state's selective B and C from a repacked copy.
inline bool stageable(const ss_fwd_params* p)
{
    return !(p->flags & (SS_B_FIXED | SS_C_FIXED | SS_COMPLEX_STATE)) && p->seqlen > 0;
}
WsLayout ws_layout(const ss_fwd_params* p, bool for_bwd)
{
    const size_t nck = ((size_t)p->seqlen + SS_CHECKPOINT_STEPS - 1) / SS_CHECKPOINT_STEPS;
    const size_t rows = (size_t)p->batch * p->dim;
    const size_t esz = p->io_dtype == SS_BF16 ? 2 : 4;
    WsLayout w{};
    w.plan = plan_segments(p->batch, p->dim, p->seqlen, p->flags);
    const size_t ns = (size_t)w.plan.nseg, split = ns > 1 ? 1 : 0;
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t at = off; off += round_up(bytes, 256); return at; };
    const size_t groups = ((size_t)slots(p) + 15) / 16;   // states are handled 16 at a time
    w.ckpt_group = nck * rows * 16 * sizeof(float);
    w.ckpt_off = take(for_bwd ? groups * w.ckpt_group : 0);
    // the pre-gate y: for the backward pass, and as the accumulator across state groups
    w.y_off = take((for_bwd || groups > 1) && (p->flags & SS_HAS_Z) ? rows * (size_t)p->seqlen * esz : 0);
    w.segh_off = take(split * ns * rows * 16 * sizeof(float));
    w.segdt_off = take(split * ns * rows * sizeof(float));
    w.segg_off = take(for_bwd ? split * ns * rows * 16 * sizeof(float) : 0);
    w.dA_off = take(for_bwd ? ns * rows * 16 * sizeof(float) : 0);
    w.dD_off = take(for_bwd ? ns * rows * sizeof(float) : 0);
    w.db_off = take(for_bwd ? ns * rows * sizeof(float) : 0);
    // per-batch partial sums of the gradient of a time-invariant B / C
    w.dBf_off = take(for_bwd && (p->flags & SS_B_FIXED) ? rows * 16 * sizeof(float) : 0);
    w.dCf_off = take(for_bwd && (p->flags & SS_C_FIXED) ? rows * 16 * sizeof(float) : 0);
    w.Lp = (p->seqlen + 31) / 32 * 32;
    w.bcs_off = take(stageable(p) ? (size_t)p->batch * (((size_t)slots(p) + 15) / 16 * 16) * w.Lp * 2 * esz : 0);
    w.total = off;
    return w;
}

int check_fwd(const ss_fwd_params* p, bool for_bwd, bool bc_dense = true)
{
    if (!p) return SS_ERR_NULL;
    if (p->batch < 1 || p->dim < 1 || p->dstate < 1 || p->seqlen < 0) return SS_ERR_SHAPE;
    if (p->dstate > SS_MAX_DSTATE || slots(p) > SS_MAX_DSTATE) return SS_ERR_UNSUPPORTED;
    if ((p->flags & SS_COMPLEX_STATE) && (p->flags & SS_EXACT_ZOH_B)) return SS_ERR_UNSUPPORTED;
    if (p->io_dtype != SS_F32 && p->io_dtype != SS_BF16) return SS_ERR_UNSUPPORTED;
    if (p->flags & ~kFwdFlags) return SS_ERR_UNSUPPORTED;
    const bool empty = p->seqlen == 0;  // tensors with a zero-length axis may be NULL
    if (!p->A) return SS_ERR_NULL;
    if (!empty && (!p->u || !p->delta || !p->Bmat || !p->Cmat)) return SS_ERR_NULL;
    if (!empty && !for_bwd && !p->out) return SS_ERR_NULL;
    if (!empty && (p->flags & SS_HAS_Z) && !p->z) return SS_ERR_NULL;
    if ((p->flags & SS_HAS_D) && !p->Dskip) return SS_ERR_NULL;
    if ((p->flags & SS_HAS_DELTA_BIAS) && !p->delta_bias) return SS_ERR_NULL;
    if ((p->flags & SS_HAS_H0) && !p->h0) return SS_ERR_NULL;
    if (!for_bwd && (p->flags & SS_WRITE_H_LAST) && !p->h_last) return SS_ERR_NULL;
    const void* io[] = {p->u, p->delta, p->z, for_bwd ? nullptr : p->out};
    for (const void* q : io)
        if (q && !aligned(q, 16)) return SS_ERR_ALIGN;
    // B and C are read 16 bytes at a time only when every row is a whole number of such pieces;
    // the layer passes rows of a larger matrix here, which then are merely element-aligned
    const size_t bc_align = (p->seqlen % 8 == 0 || bc_dense) ? 16 : (p->io_dtype == SS_BF16 ? 2 : 4);
    if (p->Bmat && !aligned(p->Bmat, (p->flags & SS_B_FIXED) ? 4 : bc_align)) return SS_ERR_ALIGN;
    if (p->Cmat && !aligned(p->Cmat, (p->flags & SS_C_FIXED) ? 4 : bc_align)) return SS_ERR_ALIGN;
    const void* f32[] = {p->A, p->Dskip, p->delta_bias, p->h0, for_bwd ? nullptr : p->h_last};
    for (const void* q : f32)
        if (q && !aligned(q, 4)) return SS_ERR_ALIGN;
    if (!for_bwd && !(p->flags & SS_SAVE_FOR_BWD) && slots(p) > 16 && (p->flags & SS_HAS_Z) && p->seqlen > 0) {
        // the pre-gate output is accumulated over the groups of 16 states in the workspace
        if (!p->workspace || p->workspace_bytes < ws_layout(p, false).total) return SS_ERR_WORKSPACE;
        if (!aligned(p->workspace, 256)) return SS_ERR_ALIGN;
    }
    if (for_bwd || (p->flags & SS_SAVE_FOR_BWD)) {
        const size_t need = ws_layout(p, true).total;
        if (!p->workspace || p->workspace_bytes < need) return SS_ERR_WORKSPACE;
        if (!aligned(p->workspace, 256)) return SS_ERR_ALIGN;
    }
    return SS_OK;
}

// Whether a pass over fewer than 16 states deals them out to the waves in turn (FwdArgs::il): the
// common path only.  Forward and backward call derive it from the same arguments.
inline bool deals_states(int vec_ok, uint32_t flags)
{
    return vec_ok && !(flags & (SS_EXACT_ZOH_B | SS_B_FIXED | SS_C_FIXED | SS_COMPLEX_STATE));
}

ss::FwdArgs make_fwd_args(const ss_fwd_params* p, long bc_bstride)
{
    ss::FwdArgs a{};
    a.B = p->batch; a.D = p->dim; a.L = p->seqlen; a.N = slots(p); a.NS = slots(p);
    a.acc_y = 0;
    a.flags = p->flags;
    // 16-byte slices, addressed through per-workgroup buffer resources (64 rows, 31-bit offsets)
    a.vec_ok = p->seqlen % 8 == 0 && (size_t)p->seqlen * 64 * sizeof(float) < ((size_t)1 << 31);
    a.il = deals_states(a.vec_ok, p->flags) && a.N < 16;
    a.u = p->u; a.delta = p->delta; a.z = (p->flags & SS_HAS_Z) ? p->z : nullptr;
    a.Bm = p->Bmat; a.Cm = p->Cmat; a.A = p->A;
    a.bc_bstride = bc_bstride;
    a.Dskip = p->Dskip; a.bias = p->delta_bias; a.h0 = p->h0;
    a.out = p->out;
    a.h_last = (p->flags & SS_WRITE_H_LAST) ? p->h_last : nullptr;
    a.ckpt = nullptr;
    a.ysave = nullptr;
    a.nseg = 1;
    a.seg_len = (p->seqlen + 31) / 32 * 32 + 32;
    a.seg_h = nullptr;
    a.seg_sumdt = nullptr;
    a.bcs = nullptr; a.Lp = 0;
    a.W_dt = nullptr; a.rT = nullptr; a.R = 0; a.Rp = 0;
    return a;
}

// Narrows the arguments of a whole call to the g-th group of 16 states: every (..., n) pointer
// moves to the group's first state (the stride stays NS), checkpoints get the group's block.
template <typename P> P* at(P* base, long elems) { return base ? base + elems : base; }
const void* at_bytes(const void* base, size_t bytes) { return base ? static_cast<const char*>(base) + bytes : base; }

void narrow_to_group(ss::FwdArgs& a, const ss_fwd_params* p, int g, size_t ckpt_group_bytes)
{
    const int n0 = g * 16;
    const size_t esz = p->io_dtype == SS_BF16 ? 2 : 4;
    a.N = slots(p) - n0 < 16 ? slots(p) - n0 : 16;
    a.il = deals_states(a.vec_ok, p->flags) && a.N < 16;
    a.A = at(a.A, n0);
    a.h0 = at(a.h0, n0);
    a.h_last = at(a.h_last, n0);
    a.Bm = (p->flags & SS_B_FIXED) ? at_bytes(a.Bm, (size_t)n0 * 4) : at_bytes(a.Bm, (size_t)n0 * p->seqlen * esz);
    a.Cm = (p->flags & SS_C_FIXED) ? at_bytes(a.Cm, (size_t)n0 * 4) : at_bytes(a.Cm, (size_t)n0 * p->seqlen * esz);
    a.bcs = at_bytes(a.bcs, (size_t)(n0 / 4) * (a.Lp / 4) * 32 * esz);   // the group's first packed piece
    if (a.ckpt) a.ckpt = reinterpret_cast<float*>(reinterpret_cast<char*>(a.ckpt) + (size_t)g * ckpt_group_bytes);
    if (g > 0) {
        a.flags &= ~(uint32_t)SS_HAS_D;   // the skip term enters once
        a.acc_y = 1;
    }
}

// Device address of `scratch` on the current device, looked up once per device.
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];
int static_scratch(void** out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SS_ERR_LAUNCH;
    void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return SS_ERR_LAUNCH;
        g_scratch_ptr[dev].store(ptr, std::memory_order_release);   // the same value from every thread
    }
    *out = ptr;
    return SS_OK;
}

}  // namespace

namespace ss {

// The fused projection exists for the plain bf16 kernel on an unsplit sequence of whole 8-step
// slices, with a workspace for the repacked operands.
bool scan_fwd_fusable(const ss_fwd_params* p, int R)
{
    if (!p || p->seqlen < 1 || p->io_dtype != SS_BF16 || !stageable(p) || slots(p) > 16) return false;
    if (R < 8 || R % 8 != 0 || R > 256 || (p->flags & SS_EXACT_ZOH_B)) return false;
    if (p->seqlen % 8 != 0 || (size_t)p->seqlen * 64 * sizeof(float) >= ((size_t)1 << 31)) return false;
    if (plan_segments(p->batch, p->dim, p->seqlen, p->flags).nseg != 1) return false;
    return p->workspace && aligned(p->workspace, 256) &&
           p->workspace_bytes >= ws_layout(p, (p->flags & SS_SAVE_FOR_BWD) != 0).total;
}

static int scan_fwd_impl(const ss_fwd_params* p, long bc_bstride, const void* W_dt, int R, const void* rT, void* stream)
{
    const int rc = check_fwd(p, false, p && bc_bstride == (long)slots(p) * p->seqlen);
    if (rc != SS_OK) return rc;
    ss::FwdArgs a = make_fwd_args(p, bc_bstride);
    if (W_dt) {
        if (!scan_fwd_fusable(p, R) || !aligned(W_dt, 16) || !aligned(rT, 16)) return SS_ERR_UNSUPPORTED;
        a.W_dt = W_dt; a.rT = rT; a.R = R; a.Rp = (R + 31) / 32 * 32;
    }
    char* ws = static_cast<char*>(p->workspace);
    const int groups = p->seqlen == 0 ? 1 : (slots(p) + 15) / 16;
    size_t ckpt_group = 0;
    // the repacked copy serves the scalar path only: sequences of whole 16-byte pieces stage B and C through LDS instead
    auto stage = [&](const WsLayout& w) {
        a.Lp = w.Lp;
        if (a.vec_ok) return true;
        if (ss::launch_stage_bc(a, ws + w.bcs_off, p->io_dtype, static_cast<hipStream_t>(stream)) != 0) return false;
        a.bcs = ws + w.bcs_off;
        return true;
    };
    if (p->flags & SS_SAVE_FOR_BWD) {
        const WsLayout w = ws_layout(p, true);
        if (stageable(p) && !stage(w)) return SS_ERR_LAUNCH;
        ckpt_group = w.ckpt_group;
        a.ckpt = reinterpret_cast<float*>(ws + w.ckpt_off);
        a.ysave = (p->flags & SS_HAS_Z) ? ws + w.y_off : nullptr;
        if (w.plan.nseg > 1) {
            a.nseg = w.plan.nseg; a.seg_len = w.plan.seg_len;
            a.seg_h = reinterpret_cast<float*>(ws + w.segh_off);
            a.seg_sumdt = reinterpret_cast<float*>(ws + w.segdt_off);
        }
    } else {
        // a plain forward call splits the sequence only if the caller lent the scratch for it
        const WsLayout w = ws_layout(p, false);
        const bool lent = ws && p->workspace_bytes >= w.total && aligned(ws, 256);
        if (stageable(p) && lent && !stage(w)) return SS_ERR_LAUNCH;
        if (groups > 1 && (p->flags & SS_HAS_Z)) a.ysave = ws + w.y_off;   // checked to be there
        if (w.plan.nseg > 1 && lent) {
            a.nseg = w.plan.nseg; a.seg_len = w.plan.seg_len;
            a.seg_h = reinterpret_cast<float*>(ws + w.segh_off);
            a.seg_sumdt = reinterpret_cast<float*>(ws + w.segdt_off);
        }
    }
    // one pass per group of 16 states; the passes run in stream order and share the segment
    // buffers, each adds its C*h to the y of the ones before it
    for (int g = 0; g < groups; ++g) {
        ss::FwdArgs ag = a;
        if (groups > 1) narrow_to_group(ag, p, g, ckpt_group);
        if (ss::launch_fwd(ag, p->io_dtype, static_cast<hipStream_t>(stream)) != 0) return SS_ERR_LAUNCH;
    }
    return SS_OK;
}


int scan_fwd_strided(const ss_fwd_params* p, long bc_bstride, void* stream)
{
    return scan_fwd_impl(p, bc_bstride, nullptr, 0, nullptr, stream);
}

int scan_fwd_fused(const ss_fwd_params* p, long bc_bstride, const void* W_dt, int R, const void* rT, void* stream)
{
    if (!W_dt || !rT) return SS_ERR_NULL;
    return scan_fwd_impl(p, bc_bstride, W_dt, R, rT, stream);
}

int scan_bwd_strided(const ss_bwd_params* p, long bc_bstride, void* stream)
{
    if (!p) return SS_ERR_NULL;
    const int rc = check_fwd(&p->fwd, true, bc_bstride == (long)slots(&p->fwd) * p->fwd.seqlen);
    if (rc != SS_OK) return rc;
    const ss_fwd_params* f = &p->fwd;
    const bool empty = f->seqlen == 0;
    if (!p->dA) return SS_ERR_NULL;
    if (!empty && (!p->dout || !p->du || !p->ddelta || !p->dB || !p->dC)) return SS_ERR_NULL;
    if (((f->flags & SS_B_FIXED) && !p->dB) || ((f->flags & SS_C_FIXED) && !p->dC)) return SS_ERR_NULL;
    if (!empty && (f->flags & SS_HAS_Z) && !p->dz) return SS_ERR_NULL;
    if ((f->flags & SS_HAS_D) && !p->dD) return SS_ERR_NULL;
    if ((f->flags & SS_HAS_DELTA_BIAS) && !p->ddelta_bias) return SS_ERR_NULL;
    const void* io[] = {p->dout, p->du, p->ddelta, p->dz};
    for (const void* q : io)
        if (q && !aligned(q, 16)) return SS_ERR_ALIGN;
    const void* f32[] = {p->dh_last, p->dB, p->dC, p->dA, p->dD, p->ddelta_bias, p->dh0};
    for (const void* q : f32)
        if (q && !aligned(q, 4)) return SS_ERR_ALIGN;

    const WsLayout w = ws_layout(f, true);
    char* ws = static_cast<char*>(f->workspace);
    ss::BwdArgs a{};
    a.f = make_fwd_args(f, bc_bstride);
    a.f.out = nullptr;
    a.f.h_last = nullptr;
    a.f.ckpt = reinterpret_cast<float*>(ws + w.ckpt_off);
    a.f.ysave = (f->flags & SS_HAS_Z) ? ws + w.y_off : nullptr;
    if (w.plan.nseg > 1) {
        a.f.nseg = w.plan.nseg; a.f.seg_len = w.plan.seg_len;
        a.f.seg_h = reinterpret_cast<float*>(ws + w.segh_off);
        a.f.seg_sumdt = reinterpret_cast<float*>(ws + w.segdt_off);
        a.seg_g = reinterpret_cast<float*>(ws + w.segg_off);
    }
    a.dout = p->dout; a.dh_last = p->dh_last;
    a.du = p->du; a.ddelta = p->ddelta; a.dz = (f->flags & SS_HAS_Z) ? p->dz : nullptr;
    a.dB = p->dB; a.dC = p->dC;
    a.dA_part = reinterpret_cast<float*>(ws + w.dA_off);
    a.dBf_part = reinterpret_cast<float*>(ws + w.dBf_off);
    a.dCf_part = reinterpret_cast<float*>(ws + w.dCf_off);
    a.dD_part = reinterpret_cast<float*>(ws + w.dD_off);
    a.db_part = reinterpret_cast<float*>(ws + w.db_off);
    a.dh0 = p->dh0;
    a.dA = p->dA;
    a.dD = (f->flags & SS_HAS_D) ? p->dD : nullptr;
    a.dbias = (f->flags & SS_HAS_DELTA_BIAS) ? p->ddelta_bias : nullptr;
    a.acc = 0;
    a.dbc_bstride = (long)slots(f) * f->seqlen;
    // one pass per group of 16 states, in stream order: each adds its share of du, ddelta and
    // dbias to the earlier ones' and writes its own slices of dA, dB, dC and dh0
    const int groups = (slots(f) + 15) / 16;
    for (int g = 0; g < groups; ++g) {
        ss::BwdArgs ag = a;
        if (groups > 1) {
            const int n0 = g * 16;
            narrow_to_group(ag.f, f, g, w.ckpt_group);
            ag.f.acc_y = 0;
            ag.acc = g > 0;
            ag.dh_last = at(ag.dh_last, n0);
            ag.dh0 = at(ag.dh0, n0);
            ag.dA = at(ag.dA, n0);
            ag.dB = at(ag.dB, (f->flags & SS_B_FIXED) ? (long)n0 : (long)n0 * f->seqlen);
            ag.dC = at(ag.dC, (f->flags & SS_C_FIXED) ? (long)n0 : (long)n0 * f->seqlen);
            if (g > 0) { ag.dz = nullptr; ag.dD = nullptr; }
        }
        if (ss::launch_bwd(ag, f->io_dtype, static_cast<hipStream_t>(stream)) != 0) return SS_ERR_LAUNCH;
    }
    return SS_OK;
}


static int step_impl(const ss_step_params* p, long bc_stride, const float* P, const void* W_dt, int R, int ldp, void* stream)
{
    if (!p) return SS_ERR_NULL;
    if (p->batch < 1 || p->dim < 1 || p->dstate < 1) return SS_ERR_SHAPE;
    if (p->dstate > SS_MAX_DSTATE || slots(p) > SS_MAX_DSTATE) return SS_ERR_UNSUPPORTED;
    if ((p->flags & SS_COMPLEX_STATE) && (p->flags & SS_EXACT_ZOH_B)) return SS_ERR_UNSUPPORTED;
    if (p->io_dtype != SS_F32 && p->io_dtype != SS_BF16) return SS_ERR_UNSUPPORTED;
    if (p->flags & ~kStepFlags) return SS_ERR_UNSUPPORTED;
    if (!p->h || !p->u_t || !p->A || !p->out_t) return SS_ERR_NULL;
    if (!P && (!p->delta_t || !p->B_t || !p->C_t)) return SS_ERR_NULL;
    if ((p->flags & SS_HAS_Z) && !p->z_t) return SS_ERR_NULL;
    if ((p->flags & SS_HAS_D) && !p->Dskip) return SS_ERR_NULL;
    if ((p->flags & SS_HAS_DELTA_BIAS) && !p->delta_bias) return SS_ERR_NULL;
    if (!aligned(p->h, 16)) return SS_ERR_ALIGN;
    const size_t esz = p->io_dtype == SS_BF16 ? 2 : 4;
    const void* io[] = {p->u_t, p->delta_t, p->z_t, p->out_t};
    for (const void* q : io)
        if (q && !aligned(q, esz)) return SS_ERR_ALIGN;
    if (!P && (!aligned(p->B_t, (p->flags & SS_B_FIXED) ? 4 : esz) || !aligned(p->C_t, (p->flags & SS_C_FIXED) ? 4 : esz)))
        return SS_ERR_ALIGN;
    if (P && (!aligned(P, 16) || !aligned(W_dt, 16) || !aligned(p->h, 16) || R % 8 != 0 || ldp % 4 != 0)) return SS_ERR_ALIGN;
    const void* f32[] = {p->A, p->Dskip, p->delta_bias};
    for (const void* q : f32)
        if (q && !aligned(q, 4)) return SS_ERR_ALIGN;
    ss::StepArgs a{};
    a.B = p->batch; a.D = p->dim; a.N = slots(p); a.flags = p->flags;
    a.h = p->h; a.u_t = p->u_t; a.delta_t = p->delta_t; a.z_t = p->z_t;
    a.B_t = P ? nullptr : p->B_t; a.C_t = P ? nullptr : p->C_t; a.bc_stride = bc_stride;
    a.P = P; a.W_dt = W_dt; a.R = R; a.ldp = ldp; a.A = p->A; a.Dskip = p->Dskip; a.bias = p->delta_bias;
    a.out_t = p->out_t;
    if (P) return ss::launch_step_projected(a, static_cast<hipStream_t>(stream)) == 0 ? SS_OK : SS_ERR_LAUNCH;
    return ss::launch_step(a, p->io_dtype, static_cast<hipStream_t>(stream)) == 0 ? SS_OK : SS_ERR_LAUNCH;
}

int step_strided(const ss_step_params* p, long bc_stride, void* stream)
{
    return step_impl(p, bc_stride, nullptr, nullptr, 0, 0, stream);
}

int step_projected(const ss_step_params* p, const float* P, const void* W_dt, int R, int ldp, void* stream)
{
    if (!p || !P || !W_dt) return SS_ERR_NULL;
    if (p->io_dtype != SS_BF16 || R > 256 || p->dstate > 16 || ldp > 256 + 2 * 16) return SS_ERR_UNSUPPORTED;
    return step_impl(p, 0, P, W_dt, R, ldp, stream);
}

}  // namespace ss

extern "C" {

size_t ss_workspace_bytes(const ss_fwd_params* p, int for_backward)
{
    if (!p || p->batch < 1 || p->dim < 1 || p->seqlen < 0) return 0;
    return ws_layout(p, for_backward != 0).total;
}

int ss_scan_fwd(const ss_fwd_params* p, void* stream)
{
    if (!p) return SS_ERR_NULL;
    return ss::scan_fwd_strided(p, (long)slots(p) * p->seqlen, stream);
}

int ss_scan_fwd_static(const ss_fwd_params* p, void* stream)
{
    if (!p) return SS_ERR_NULL;
    if (p->flags & SS_SAVE_FOR_BWD) return SS_ERR_UNSUPPORTED;
    ss_fwd_params q = *p;
    q.workspace = nullptr;
    q.workspace_bytes = 0;
    // everything else is checked first, so that an invalid call reports its own error
    const int rc = check_fwd(&q, false);
    if (rc != SS_OK && rc != SS_ERR_WORKSPACE) return rc;
    if (ws_layout(&q, false).total > (size_t)SS_STATIC_SCRATCH_BYTES) return SS_ERR_WORKSPACE;
    void* ptr = nullptr;
    const int rs = static_scratch(&ptr);
    if (rs != SS_OK) return rs;
    q.workspace = ptr;
    q.workspace_bytes = SS_STATIC_SCRATCH_BYTES;
    return ss::scan_fwd_strided(&q, (long)slots(&q) * q.seqlen, stream);
}

int ss_scan_bwd(const ss_bwd_params* p, void* stream)
{
    if (!p) return SS_ERR_NULL;
    return ss::scan_bwd_strided(p, (long)slots(&p->fwd) * p->fwd.seqlen, stream);
}

int ss_step(const ss_step_params* p, void* stream)
{
    if (!p) return SS_ERR_NULL;
    return ss::step_strided(p, slots(p), stream);
}

const char* ss_strerror(int code)
{
    switch (code) {
    case SS_OK: return "success";
    case SS_ERR_NULL: return "a required pointer is NULL";
    case SS_ERR_SHAPE: return "batch, dim and dstate must be >= 1 and seqlen >= 0";
    case SS_ERR_UNSUPPORTED: return "unsupported dstate, io_dtype or flag";
    case SS_ERR_ALIGN: return "a pointer is not aligned as required";
    case SS_ERR_WORKSPACE: return "workspace missing or too small";
    case SS_ERR_LAUNCH: return "the HIP runtime refused a kernel launch";
    case SS_ERR_BACKEND: return "backend failure (reserved; not returned by any current entry point)";
    default: return "unknown error code";
    }
}

int ss_version(void) { return 100; }

}  // extern "C"
