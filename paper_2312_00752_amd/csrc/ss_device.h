// Device-side helpers shared by the selective-scan kernels (gfx950 only).
//
// Work decomposition used by every scan kernel in this library.  A workgroup of NWAVES
// waves owns ROWS (b,d) rows of one batch entry and walks the sequence in chunks of
// CHUNK_T steps.  In the "state view" lane l of every wave is row l, and wave w carries
// states 4w..4w+3 of that row in registers: the recurrence of Eq. 2a runs as a plain
// sequential loop with the minimum per-(t,n) work (one exp, three multiply-adds), no scan
// re-association overhead, and -- because all lanes of a wave share b, t and n -- B and C
// are wave-uniform and come through the scalar data path instead of LDS.  In the
// "pointwise view" thread i is (row i/4, 8-step slice i%4): it does the per-(b,d,t) work
// (softplus, gate, conversions) on coalesced 16-byte global accesses.  The two views
// exchange data through LDS tiles of ROWS x CHUNK_T floats.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ss {

constexpr int WAVE = 64;
constexpr int STATES_PER_LANE = 4;
constexpr int NWAVES = 4;                              // covers N <= 16
constexpr int ROWS = WAVE;                             // rows per workgroup
constexpr int THREADS = NWAVES * WAVE;                 // 256
constexpr int NPAD = STATES_PER_LANE * NWAVES;         // 16
constexpr int CHUNK_T = 32;                            // steps per forward chunk
constexpr int CKPT_T = 16;                             // == SS_CHECKPOINT_STEPS
constexpr int SLICE = CHUNK_T * ROWS / THREADS;        // 8 steps per thread in the pointwise view
constexpr int SLICES = CHUNK_T / SLICE;                // 4 threads per row in the pointwise view
constexpr int TPAD = CHUNK_T + 4;                      // LDS row pitch (floats) of (row, t) tiles

// State held by slot k of wave w, and state stored at position 4w + k of a 16-float workspace
// record: 4w + k, or 4k + w when the states are dealt out to the waves in turn (FwdArgs::il).
__host__ __device__ __forceinline__ int slot_state(int w, int k, int il) { return il ? k * NWAVES + w : w * STATES_PER_LANE + k; }
__host__ __device__ __forceinline__ int position_state(int pos, int il) { return slot_state(pos / STATES_PER_LANE, pos % STATES_PER_LANE, il); }
// slots per lane a kernel is built for when the states are dealt out: 1, 2 or 4
__host__ __device__ __forceinline__ int slots_for(int N, int il) { return !il ? STATES_PER_LANE : (N <= NWAVES ? 1 : (N <= 2 * NWAVES ? 2 : STATES_PER_LANE)); }

constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

typedef uint16_t bf16_t;  // storage only; arithmetic is always float
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float log2_fast(float x) { return __builtin_amdgcn_logf(x); }
__device__ __forceinline__ float rcp_fast(float x) { return __builtin_amdgcn_rcpf(x); }

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(uint32_t(v) << 16); }

// float -> bf16 with the hardware converter of gfx950 (round to nearest even, NaN kept)
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));  // v_cvt_pk_bf16_f32
}
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) { return pack_bf16x2(f, 0.0f) & 0xffffu; }

// softplus(r) = log(1 + e^r) and sigmoid(r), sharing one exponential and one reciprocal.
// With w = fl(1 + e) and c = e - (w - 1), the exact rounding error of that sum,
// log(1 + e) = log(w) + log(1 + c / w) = log(w) + c / w to float precision: accurate for every
// e, however small, with no case split (w = 1 gives e itself).  Above r = 20 softplus(r) = r to
// float precision (and e^r may overflow, which the select discards); the exponent is capped
// so that the sigmoid comes out as 1 there instead of inf * 0.
__device__ __forceinline__ void softplus_sigmoid(float r, float& sp, float& sg)
{
    const float e = exp2_fast(fminf(r * LOG2E, 64.0f));
    const float w = 1.0f + e;
    const float inv = rcp_fast(w);                 // 1 / (1 + e^r)
    const float c = e - (w - 1.0f);
    const float lp = fmaf(log2_fast(w), LN2, c * inv);
    sp = (r > 20.0f) ? r : lp;
    sg = e * inv;                                  // e^r / (1 + e^r)
}
// Exact zero-order hold (Eq. 4): phi(dt, A) = (exp(dt A) - 1) / A multiplies B u in the
// state update (dt itself where A == 0), and d phi / d A = (x e^x - (e^x - 1)) / A^2 with
// x = dt A (dt^2 / 2 where A == 0).  Both differences cancel for small x, where the Taylor
// series is used instead (|x| < 1/8: truncation error below 1e-8 relative).
struct zoh_terms { float phi, dphi_dA; };
__device__ __forceinline__ zoh_terms zoh_phi(float dt, float A, float invA, float abar, bool want_dA)
{
    const float x = dt * A;
    const bool small = fabsf(x) < 0.125f;
    const float em1_series = x * fmaf(x, fmaf(x, fmaf(x, fmaf(x, 1.0f / 120.0f, 1.0f / 24.0f), 1.0f / 6.0f), 0.5f), 1.0f);
    const float em1 = small ? em1_series : abar - 1.0f;
    zoh_terms r;
    r.phi = (A == 0.0f) ? dt : em1 * invA;
    r.dphi_dA = 0.0f;
    if (want_dA) {
        // x e^x - (e^x - 1) = sum_{k>=2} (k-1)/k! x^k
        const float x2 = x * x;
        const float num_series = x2 * fmaf(x, fmaf(x, fmaf(x, fmaf(x, 1.0f / 144.0f, 1.0f / 30.0f), 0.125f), 1.0f / 3.0f), 0.5f);
        const float num = small ? num_series : fmaf(x, abar, -em1);
        r.dphi_dA = (A == 0.0f) ? 0.5f * dt * dt : num * invA * invA;
    }
    return r;
}

// The same phi for the kernels that are short of registers and issue slots, from what the recurrence has
// anyway (x2 = dt A log2 e, abar = 2^x2) and inv_A = 1/A (0 for A = 0): dt (1 + x/2 + x^2/6) for
// |dt A| < 2^-7 (relative error < 3e-8; covers A = 0), (abar - 1)/A beyond (relative error of the
// exponential's last bit over |dt A|, < 2e-5).
constexpr float ZOH_SMALL_X2 = 0.0078125f * LOG2E;   // the threshold on dt * A * log2(e)
constexpr float ZOH_SMALL_X2_GRAD = 0.0625f * LOG2E;  // the same for the gradient term that carries dphi/dA (backward pass)
// |x| < limit ? small : large, as a compare and a select.  Written out: from the conditional expression the
// compiler builds a divergent branch per state and step (both sides under execution masks), which breaks an
// unrolled sweep into hundreds of basic blocks and spills hundreds of registers.
__device__ __forceinline__ float select_small(float x, float limit, float small, float large)
{
    float r;
    asm("v_cmp_lt_f32_e64 vcc, |%1|, %2\n\t"
        "v_cndmask_b32_e32 %0, %4, %3, vcc"
        : "=v"(r) : "v"(x), "s"(limit), "v"(small), "v"(large) : "vcc");
    return r;
}
__device__ __forceinline__ float zoh_phi_fast(float dt, float x2, float abar, float inv_A)
{
    const float series = dt * fmaf(x2, fmaf(x2, LN2 * LN2 / 6.0f, LN2 / 2.0f), 1.0f);
    return select_small(x2, ZOH_SMALL_X2, series, (abar - 1.0f) * inv_A);
}

// Complex decay factor of one step, abar = exp(dt (Ar + i Ai)) = (re, im): the magnitude from
// the exponential unit, the rotation from the hardware sine / cosine, which take their
// argument in revolutions (the fraction is taken first; they are specified for |x| <= 256).
struct cplx { float re, im; };
constexpr float INV_2PI = 0.15915494309189535f;
__device__ __forceinline__ cplx complex_decay(float dt, float Ar_log2e, float Ai)
{
    const float mag = exp2_fast(dt * Ar_log2e);
    const float rev = __builtin_amdgcn_fractf(dt * Ai * INV_2PI);
    cplx r;
    r.re = mag * __builtin_amdgcn_cosf(rev);
    r.im = mag * __builtin_amdgcn_sinf(rev);
    return r;
}

__device__ __forceinline__ float sigmoid_fast(float z)
{
    return rcp_fast(1.0f + exp2_fast(-z * LOG2E));
}

// A 16-byte load of data the kernel reads exactly once, with the streaming (non-temporal)
// hint.  When the row pitch is a large power of two, the rows a wave reads at the same
// step fall into the same set of the vector L1 and evict each other; streaming loads do
// not suffer from that (measured: 20 % on the forward pass of the 2^20-step workload, and
// no change where the pitch is small).  The 8-byte bf16 loads of the backward kernel keep
// the default policy: two of them share a 16-byte neighbourhood and do profit from the L1.
__device__ __forceinline__ uint4 load16_once(const void* p)
{
    const u32x4 x = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    return make_uint4(x.x, x.y, x.z, x.w);
}

// ---- workgroup numbering ---------------------------------------------------------------
// The dispatcher hands consecutive workgroup indices to the chip's eight XCDs in turn, and each
// XCD has an L2 of its own.  Renumbered like this, XCD x works on indices [x*n/8, (x+1)*n/8):
// neighbours in the index (row groups of one batch entry) share an L2.  A bijection on [0, n)
// whenever it applies (n a multiple of 8); the identity otherwise.
__device__ __forceinline__ unsigned xcd_contiguous(unsigned i, unsigned n)
{
    return (n % 8u == 0u) ? (i % 8u) * (n / 8u) + i / 8u : i;
}

// ---- buffer-addressed accesses ---------------------------------------------------------
// Memory operations retire in order and the compiler can let younger ones stay outstanding
// across a wait only if it can count them: a store or load inside an `if` counts as "maybe
// zero", and a wait for an older load then degenerates to "wait for everything", i.e. for
// the acknowledgement of stores issued a moment ago.  The hot loops therefore use buffer
// instructions, which are issued unconditionally: the hardware drops a store, and returns
// zero for a load, whose offset lies at or beyond the resource's size, so a lane (or a whole
// access) is switched off with an out-of-range offset (or a size of zero) instead of a
// branch.  Resources are built per workgroup (64 rows), which keeps offsets far below 2^31.
using rsrc_t = __amdgpu_buffer_rsrc_t;
constexpr uint32_t BUF_OFF = 0x80000000u;   // an offset beyond any resource built here
__device__ __forceinline__ rsrc_t make_rsrc(const void* p, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ uint4 buf_load16_once(rsrc_t r, uint32_t off)   // streaming hint, as load16_once
{
    const u32x4 x = __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, 2);
    return make_uint4(x.x, x.y, x.z, x.w);
}
__device__ __forceinline__ void buf_store16(rsrc_t r, uint32_t off, uint4 v)
{
    const u32x4 x = {v.x, v.y, v.z, v.w};
    __builtin_amdgcn_raw_buffer_store_b128(x, r, (int)off, 0, 0);
}

__device__ __forceinline__ uint4 buf_load16(rsrc_t r, uint32_t off)
{
    const u32x4 x = __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, 0);
    return make_uint4(x.x, x.y, x.z, x.w);
}
typedef uint32_t u32x2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint2 buf_load8(rsrc_t r, uint32_t off)
{
    const u32x2v x = __builtin_amdgcn_raw_buffer_load_b64(r, (int)off, 0, 0);
    return make_uint2(x.x, x.y);
}
// one io element as raw bits (zero if off is out of range)
template <typename T>
__device__ __forceinline__ uint32_t buf_load_elem(rsrc_t r, uint32_t off)
{
    if constexpr (sizeof(T) == 2) return (uint32_t)(unsigned short)__builtin_amdgcn_raw_buffer_load_b16(r, (int)off, 0, 0);
    else return (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(r, (int)off, 0, 0);
}

// ---- 8 consecutive io elements <-> 8 floats -------------------------------------------
// VEC: every row starts 16-byte aligned and L is a multiple of 8, so a slice is either
// whole (nvalid == 8, one or two 16-byte accesses) or empty.  Otherwise the `nvalid`
// leading elements are accessed one by one; the rest read as zero / are not written.
template <typename T> struct io8;

template <> struct io8<float> {
    struct raw { float4 a, b; };
    template <bool VEC>
    static __device__ __forceinline__ raw load(const float* p, int nvalid)
    {
        raw r;
        if (VEC) {  // nvalid is 0 or 8
            r.a = r.b = make_float4(0.f, 0.f, 0.f, 0.f);
            if (nvalid == 8) {
                const uint4 x = load16_once(p), y = load16_once(p + 4);
                r.a = make_float4(__uint_as_float(x.x), __uint_as_float(x.y), __uint_as_float(x.z), __uint_as_float(x.w));
                r.b = make_float4(__uint_as_float(y.x), __uint_as_float(y.y), __uint_as_float(y.z), __uint_as_float(y.w));
            }
        } else {
            float v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = (j < nvalid) ? p[j] : 0.0f;
            r.a = make_float4(v[0], v[1], v[2], v[3]);
            r.b = make_float4(v[4], v[5], v[6], v[7]);
        }
        return r;
    }
    static __device__ __forceinline__ raw load_buf(rsrc_t rs, uint32_t off)   // whole slice, or zeros if off is out of range
    {
        const uint4 x = buf_load16_once(rs, off), y = buf_load16_once(rs, off + 16);
        raw r;
        r.a = make_float4(__uint_as_float(x.x), __uint_as_float(x.y), __uint_as_float(x.z), __uint_as_float(x.w));
        r.b = make_float4(__uint_as_float(y.x), __uint_as_float(y.y), __uint_as_float(y.z), __uint_as_float(y.w));
        return r;
    }
    struct packed { uint4 a, b; };   // eight elements as stored
    static __device__ __forceinline__ packed pack(const float (&v)[8])
    {
        return {make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])),
                make_uint4(__float_as_uint(v[4]), __float_as_uint(v[5]), __float_as_uint(v[6]), __float_as_uint(v[7]))};
    }
    static __device__ __forceinline__ void store_packed(rsrc_t rs, uint32_t off, const packed& x)   // dropped if off is out of range
    {
        buf_store16(rs, off, x.a);
        buf_store16(rs, off + 16, x.b);
    }
    static __device__ __forceinline__ void store_buf(rsrc_t rs, uint32_t off, const float (&v)[8]) { store_packed(rs, off, pack(v)); }
    static __device__ __forceinline__ void unpack(const raw& r, float (&v)[8])
    {
        v[0] = r.a.x; v[1] = r.a.y; v[2] = r.a.z; v[3] = r.a.w;
        v[4] = r.b.x; v[5] = r.b.y; v[6] = r.b.z; v[7] = r.b.w;
    }
    template <bool VEC>
    static __device__ __forceinline__ void store(float* p, const float (&v)[8], int nvalid)
    {
        if (VEC) {
            if (nvalid == 8) {
                *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
                *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
            }
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (j < nvalid) p[j] = v[j];
        }
    }
};

template <> struct io8<bf16_t> {
    struct raw { uint4 w; };
    template <bool VEC>
    static __device__ __forceinline__ raw load(const bf16_t* p, int nvalid)
    {
        raw r;
        if (VEC) {  // nvalid is 0 or 8
            r.w = make_uint4(0u, 0u, 0u, 0u);
            if (nvalid == 8) r.w = load16_once(p);
        } else {
            uint32_t v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = (j < nvalid) ? uint32_t(p[j]) : 0u;
            r.w = make_uint4(v[0] | (v[1] << 16), v[2] | (v[3] << 16), v[4] | (v[5] << 16),
                             v[6] | (v[7] << 16));
        }
        return r;
    }
    static __device__ __forceinline__ raw load_buf(rsrc_t rs, uint32_t off)   // whole slice, or zeros if off is out of range
    {
        raw r;
        r.w = buf_load16_once(rs, off);
        return r;
    }
    typedef uint4 packed;   // eight elements as stored
    static __device__ __forceinline__ packed pack(const float (&v)[8])
    {
        return make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7]));
    }
    static __device__ __forceinline__ void store_packed(rsrc_t rs, uint32_t off, packed x) { buf_store16(rs, off, x); }   // dropped if off is out of range
    static __device__ __forceinline__ void store_buf(rsrc_t rs, uint32_t off, const float (&v)[8]) { store_packed(rs, off, pack(v)); }
    static __device__ __forceinline__ void unpack(const raw& r, float (&v)[8])
    {
        v[0] = bf16_lo(r.w.x); v[1] = bf16_hi(r.w.x);
        v[2] = bf16_lo(r.w.y); v[3] = bf16_hi(r.w.y);
        v[4] = bf16_lo(r.w.z); v[5] = bf16_hi(r.w.z);
        v[6] = bf16_lo(r.w.w); v[7] = bf16_hi(r.w.w);
    }
    template <bool VEC>
    static __device__ __forceinline__ void store(bf16_t* p, const float (&v)[8], int nvalid)
    {
        if (VEC) {
            if (nvalid == 8)
                *reinterpret_cast<uint4*>(p) = make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]),
                                                          pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7]));
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (j < nvalid) p[j] = bf16_t(f32_to_bf16_bits(v[j]));
        }
    }
};

// ---- 4 consecutive io elements <-> 4 floats (same VEC contract: whole or empty) ----------
template <typename T> struct io4;

template <> struct io4<float> {
    struct raw { float4 a; };
    template <bool VEC>
    static __device__ __forceinline__ raw load(const float* p, int nvalid)
    {
        raw r;
        if (VEC) {
            r.a = make_float4(0.f, 0.f, 0.f, 0.f);
            if (nvalid == 4) {
                const uint4 x = load16_once(p);
                r.a = make_float4(__uint_as_float(x.x), __uint_as_float(x.y), __uint_as_float(x.z), __uint_as_float(x.w));
            }
        } else {
            r.a = make_float4(0 < nvalid ? p[0] : 0.f, 1 < nvalid ? p[1] : 0.f, 2 < nvalid ? p[2] : 0.f,
                              3 < nvalid ? p[3] : 0.f);
        }
        return r;
    }
    static __device__ __forceinline__ raw load_buf(rsrc_t rs, uint32_t off)   // whole slice, or zeros if off is out of range
    {
        const uint4 x = buf_load16(rs, off);
        raw r;
        r.a = make_float4(__uint_as_float(x.x), __uint_as_float(x.y), __uint_as_float(x.z), __uint_as_float(x.w));
        return r;
    }
    typedef uint4 packed;   // four elements as stored
    static __device__ __forceinline__ packed pack(const float (&v)[4])
    {
        return make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3]));
    }
    static __device__ __forceinline__ void store_packed(rsrc_t rs, uint32_t off, packed x) { buf_store16(rs, off, x); }   // dropped if off is out of range
    static __device__ __forceinline__ void store_buf(rsrc_t rs, uint32_t off, const float (&v)[4]) { store_packed(rs, off, pack(v)); }
    static __device__ __forceinline__ void unpack(const raw& r, float (&v)[4])
    {
        v[0] = r.a.x; v[1] = r.a.y; v[2] = r.a.z; v[3] = r.a.w;
    }
    template <bool VEC>
    static __device__ __forceinline__ void store(float* p, const float (&v)[4], int nvalid)
    {
        if (VEC) {
            if (nvalid == 4) *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (j < nvalid) p[j] = v[j];
        }
    }
};

template <> struct io4<bf16_t> {
    struct raw { uint2 w; };
    template <bool VEC>
    static __device__ __forceinline__ raw load(const bf16_t* p, int nvalid)
    {
        raw r;
        if (VEC) {
            r.w = make_uint2(0u, 0u);
            if (nvalid == 4) r.w = *reinterpret_cast<const uint2*>(p);
        } else {
            uint32_t v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = (j < nvalid) ? uint32_t(p[j]) : 0u;
            r.w = make_uint2(v[0] | (v[1] << 16), v[2] | (v[3] << 16));
        }
        return r;
    }
    static __device__ __forceinline__ raw load_buf(rsrc_t rs, uint32_t off)   // whole slice, or zeros if off is out of range
    {
        raw r;
        r.w = buf_load8(rs, off);
        return r;
    }
    typedef uint2 packed;   // four elements as stored
    static __device__ __forceinline__ packed pack(const float (&v)[4]) { return make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])); }
    static __device__ __forceinline__ void store_packed(rsrc_t rs, uint32_t off, packed p)   // dropped if off is out of range
    {
        const u32x2v x = {p.x, p.y};
        __builtin_amdgcn_raw_buffer_store_b64(x, rs, (int)off, 0, 0);
    }
    static __device__ __forceinline__ void store_buf(rsrc_t rs, uint32_t off, const float (&v)[4]) { store_packed(rs, off, pack(v)); }
    static __device__ __forceinline__ void unpack(const raw& r, float (&v)[4])
    {
        v[0] = bf16_lo(r.w.x); v[1] = bf16_hi(r.w.x);
        v[2] = bf16_lo(r.w.y); v[3] = bf16_hi(r.w.y);
    }
    template <bool VEC>
    static __device__ __forceinline__ void store(bf16_t* p, const float (&v)[4], int nvalid)
    {
        if (VEC) {
            if (nvalid == 4)
                *reinterpret_cast<uint2*>(p) = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (j < nvalid) p[j] = bf16_t(f32_to_bf16_bits(v[j]));
        }
    }
};

__device__ __forceinline__ float f4_get(const float4& v, int j)
{
    return j == 0 ? v.x : (j == 1 ? v.y : (j == 2 ? v.z : v.w));
}

// ---- wave-uniform fetch of B or C for one state over a group of GROUP_T steps ------------
// The address depends only on the block, the wave index and loop counters, so the load
// and the bf16 widening are done by the scalar unit and the values reach the vector ALU
// as scalar operands.  Groups are kept small (4 steps: 8 or 16 bytes) so that two groups
// of all 8 (state, B|C) rows fit the scalar register file and the next group can be in
// flight while the current one is consumed.
constexpr int GROUP_T = 4;
typedef __attribute__((address_space(4))) const u32x2 const_u32x2;  // constant address space
typedef __attribute__((address_space(4))) const u32x4 const_u32x4;

template <typename T> struct bc_group;
template <> struct bc_group<float> {
    uint32_t w[4];
    __device__ __forceinline__ float get(int j) const { return __uint_as_float(w[j]); }
};
template <> struct bc_group<bf16_t> {
    uint32_t w[2];
    __device__ __forceinline__ float get(int j) const { return (j & 1) ? bf16_hi(w[j >> 1]) : bf16_lo(w[j >> 1]); }
};

// p: start of the (b,n) row; t: first step of the group; L: row length.
// MASKED: `state_ok` false (padding state) reads as zero.
template <typename T, bool VEC, bool MASKED>
__device__ __forceinline__ bc_group<T> load_bc(const T* __restrict__ p, int t, int L, bool state_ok)
{
    bc_group<T> g;
    if (VEC) {
        // Rows are 16-byte aligned and L is a multiple of 8, so a group is whole or lies
        // entirely past the end; the latter is redirected to the last whole group (its
        // values are never used: those steps run with dt = 0 and are not stored).  B and
        // C are never written by the kernels, so reading them through the constant address
        // space is sound; with the wave-uniform address it selects the scalar load path.
        const int tc = min(t, L - GROUP_T);
        if constexpr (sizeof(T) == 2) {
            const u32x2 v = *(const_u32x2*)(p + tc);
            g.w[0] = v.x; g.w[1] = v.y;
        } else {
            const u32x4 v = *(const_u32x4*)(p + tc);
            g.w[0] = v.x; g.w[1] = v.y; g.w[2] = v.z; g.w[3] = v.w;
        }
        if (MASKED) {
#pragma unroll
            for (int i = 0; i < int(sizeof(g.w) / 4); ++i) g.w[i] = state_ok ? g.w[i] : 0u;
        }
    } else {
        uint32_t e[GROUP_T];
#pragma unroll
        for (int j = 0; j < GROUP_T; ++j) {
            const bool ok = (!MASKED || state_ok) && (t + j < L);
            if constexpr (sizeof(T) == 2) e[j] = ok ? uint32_t(p[t + j]) : 0u;
            else e[j] = ok ? __float_as_uint(p[t + j]) : 0u;
        }
        if constexpr (sizeof(T) == 2) { g.w[0] = e[0] | (e[1] << 16); g.w[1] = e[2] | (e[3] << 16); }
        else { g.w[0] = e[0]; g.w[1] = e[1]; g.w[2] = e[2]; g.w[3] = e[3]; }
    }
    return g;
}

// The same from the staged, wave-packed copy (see stage_bc_kernel): everything a wave needs of
// B and C for one group of steps is one contiguous piece, element (which * 4 + k) * 4 + j for
// B (which = 0) or C (1), the wave's state k and step j.  One or two scalar loads, no clamp,
// no mask, one base address per wave.
typedef uint32_t u32x16 __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(4))) const u32x16 const_u32x16;
constexpr int STAGE_GROUP = 2 * STATES_PER_LANE * GROUP_T;   // elements per wave and group
template <typename T> struct bcs_group;
template <> struct bcs_group<float> {
    uint32_t w[STAGE_GROUP];
    __device__ __forceinline__ float B(int k, int j) const { return __uint_as_float(w[k * GROUP_T + j]); }
    __device__ __forceinline__ float C(int k, int j) const { return __uint_as_float(w[(STATES_PER_LANE + k) * GROUP_T + j]); }
};
template <> struct bcs_group<bf16_t> {
    uint32_t w[STAGE_GROUP / 2];
    __device__ __forceinline__ float get(int e) const { return (e & 1) ? bf16_hi(w[e >> 1]) : bf16_lo(w[e >> 1]); }
    __device__ __forceinline__ float B(int k, int j) const { return get(k * GROUP_T + j); }
    __device__ __forceinline__ float C(int k, int j) const { return get((STATES_PER_LANE + k) * GROUP_T + j); }
};
template <typename T>
__device__ __forceinline__ bcs_group<T> load_bcs(const T* __restrict__ p)
{
    bcs_group<T> g;
    const u32x16 v = *(const_u32x16*)p;
#pragma unroll
    for (int i = 0; i < 16; ++i) g.w[i] = v[i];
    if constexpr (sizeof(T) == 4) {
        const u32x16 v2 = *(const_u32x16*)(p + 16);
#pragma unroll
        for (int i = 0; i < 16; ++i) g.w[16 + i] = v2[i];
    }
    return g;
}

// The scalar loads above are issued only one group (4 steps) ahead, which hides an L2 hit
// but not a trip to HBM.  When B and C are not already L2-resident (one batch entry, long
// sequence), the wave therefore touches the lines it will need one chunk later with
// ordinary vector loads: lanes 0..3 one element of each of its B rows, lanes 4..7 of its C
// rows, at step t.  The value is only handed to `consume_touch` an iteration later.
template <typename T>
__device__ __forceinline__ uint32_t touch_bc(const void* Bm, const void* Cm, int b, long bstride, int N, int L, int w,
                                              int lane, int t)
{
    // the raw bits, untouched: any arithmetic on the value would make the wave wait for it here
    uint32_t v = 0u;
    if (lane < 2 * STATES_PER_LANE && t >= 0 && t < L) {
        const int n = min(w * STATES_PER_LANE + (lane & 3), N - 1);
        const T* p = static_cast<const T*>(lane < STATES_PER_LANE ? Bm : Cm) + (long)b * bstride + (long)n * L + t;
        if constexpr (sizeof(T) == 2) v = *p; else v = __float_as_uint(*p);
    }
    return v;
}
// Rows of the pointwise view.  Four lanes share a row (one 16-byte piece of it each, or two), so sixteen
// consecutive lanes - what the LDS serves together - hold four rows.  With consecutive rows and the padded
// pitches that keep the one-lane-per-row view free of bank conflicts (five or nine pieces per row), those
// sixteen lanes collided two-way (3-4 % of the backward kernel's time); with the rows picked as below they
// touch sixteen different 16-byte slots.  A wave still owns sixteen consecutive rows, and the four lanes of
// a row stay adjacent, so global accesses do not change.
//   pitch 5, one piece per lane  (slot = 5 r + q):      rows r, r + 4, r + 8, r + 12
//   pitch 9, pieces 2 q, 2 q + 1 (slot = 9 r + 2 q):    rows r, r + 1, r + 8, r + 9   (r even)
__device__ __forceinline__ int pointwise_row_pitch5(int tid)
{
    return (tid >> 6) * 16 + ((tid >> 2) & 3) * 4 + ((tid >> 4) & 3);
}
__device__ __forceinline__ int pointwise_row_pitch9(int tid)
{
    const int m = (tid >> 2) & 3;
    return (tid >> 6) * 16 + 2 * ((tid >> 4) & 3) + (m & 1) + 8 * (m >> 1);
}
__device__ __forceinline__ void consume_touch(uint32_t v) { asm volatile("" ::"v"(v)); }

// ---- B and C as quad-broadcast operands ---------------------------------------------------
// A register that holds, in every group of four lanes, B (or C) of a wave's four state slots (slot k
// in lane k) can be the first operand of a multiply or multiply-add with the DPP control
// quad_perm [k,k,k,k]: every lane then reads slot k's value.  The compiler folds such a broadcast
// into a multiply only now and then and never into a multiply-add with an accumulator, so these
// instruction groups are written out.
typedef float f32x4_t __attribute__((ext_vector_type(4)));

// The input term of Eq. 2a for a lane's SPL states: bu[k] = B_k * du, with Bq holding B of the
// wave's states in every group of four lanes (slot k in lane k).  Written out for the same
// reason as adjoint_step_dpp, with the same leading wait state.
#define SS_QP(k) " quad_perm:[" #k "," #k "," #k "," #k "] row_mask:0xf bank_mask:0xf"
template <int SPL>
__device__ __forceinline__ void input_step_dpp(float (&bu)[STATES_PER_LANE], float Bq, float du)
{
    if constexpr (SPL == 4)
        asm("s_nop 1\n\t"
            "v_mul_f32_dpp %0, %4, %5" SS_QP(0) "\n\t"
            "v_mul_f32_dpp %1, %4, %5" SS_QP(1) "\n\t"
            "v_mul_f32_dpp %2, %4, %5" SS_QP(2) "\n\t"
            "v_mul_f32_dpp %3, %4, %5" SS_QP(3)
            : "=&v"(bu[0]), "=&v"(bu[1]), "=&v"(bu[2]), "=&v"(bu[3]) : "v"(Bq), "v"(du));
    else if constexpr (SPL == 2)
        asm("s_nop 1\n\t"
            "v_mul_f32_dpp %0, %2, %3" SS_QP(0) "\n\t"
            "v_mul_f32_dpp %1, %2, %3" SS_QP(1)
            : "=&v"(bu[0]), "=&v"(bu[1]) : "v"(Bq), "v"(du));
    else
        asm("s_nop 1\n\t"
            "v_mul_f32_dpp %0, %1, %2" SS_QP(0)
            : "=&v"(bu[0]) : "v"(Bq), "v"(du));
}

// One step of the adjoint recurrence for a lane's SPL states.  On entry g[k] = abar+ g+ of slot k;
// Cq / Bq hold C / B of the wave's states in every group of four lanes (slot k in lane k).
//     g[k] += C_k dy            (the gradient reaching h_t)          sb = sum_k B_k g[k]
// The leading wait state covers a DPP operand the compiler might have copied with a vector move
// just before (a DPP read needs two wait states after a vector write of the same register).
template <int SPL>
__device__ __forceinline__ void adjoint_step_dpp(f32x4_t& g, float& sb, float Cq, float Bq, float dy)
{
    float g0 = g[0], g1 = g[1], g2 = g[2], g3 = g[3];
    if constexpr (SPL == 4)
        asm("s_nop 1\n\t"
            "v_fmac_f32_dpp %0, %5, %7" SS_QP(0) "\n\t"
            "v_fmac_f32_dpp %1, %5, %7" SS_QP(1) "\n\t"
            "v_fmac_f32_dpp %2, %5, %7" SS_QP(2) "\n\t"
            "v_fmac_f32_dpp %3, %5, %7" SS_QP(3) "\n\t"
            "v_mul_f32_dpp %4, %6, %0" SS_QP(0) "\n\t"
            "v_fmac_f32_dpp %4, %6, %1" SS_QP(1) "\n\t"
            "v_fmac_f32_dpp %4, %6, %2" SS_QP(2) "\n\t"
            "v_fmac_f32_dpp %4, %6, %3" SS_QP(3)
            : "+v"(g0), "+v"(g1), "+v"(g2), "+v"(g3), "=&v"(sb) : "v"(Cq), "v"(Bq), "v"(dy));
    else if constexpr (SPL == 2)
        asm("s_nop 1\n\t"
            "v_fmac_f32_dpp %0, %3, %5" SS_QP(0) "\n\t"
            "v_fmac_f32_dpp %1, %3, %5" SS_QP(1) "\n\t"
            "v_mul_f32_dpp %2, %4, %0" SS_QP(0) "\n\t"
            "v_fmac_f32_dpp %2, %4, %1" SS_QP(1)
            : "+v"(g0), "+v"(g1), "=&v"(sb) : "v"(Cq), "v"(Bq), "v"(dy));
    else
        asm("s_nop 1\n\t"
            "v_fmac_f32_dpp %0, %2, %4" SS_QP(0) "\n\t"
            "v_mul_f32_dpp %1, %3, %0" SS_QP(0)
            : "+v"(g0), "=&v"(sb) : "v"(Cq), "v"(Bq), "v"(dy));
    g[0] = g0; g[1] = g1; g[2] = g2; g[3] = g3;
}
// The first half of adjoint_step_dpp alone (for the adjoint aggregate of a segment): g[k] += C_k dy.
template <int SPL>
__device__ __forceinline__ void adjoint_input_dpp(float (&g)[STATES_PER_LANE], float Cq, float dy)
{
    if constexpr (SPL == 4)
        asm("s_nop 1\n\t"
            "v_fmac_f32_dpp %0, %4, %5" SS_QP(0) "\n\t"
            "v_fmac_f32_dpp %1, %4, %5" SS_QP(1) "\n\t"
            "v_fmac_f32_dpp %2, %4, %5" SS_QP(2) "\n\t"
            "v_fmac_f32_dpp %3, %4, %5" SS_QP(3)
            : "+v"(g[0]), "+v"(g[1]), "+v"(g[2]), "+v"(g[3]) : "v"(Cq), "v"(dy));
    else if constexpr (SPL == 2)
        asm("s_nop 1\n\t"
            "v_fmac_f32_dpp %0, %2, %3" SS_QP(0) "\n\t"
            "v_fmac_f32_dpp %1, %2, %3" SS_QP(1)
            : "+v"(g[0]), "+v"(g[1]) : "v"(Cq), "v"(dy));
    else
        asm("s_nop 1\n\t"
            "v_fmac_f32_dpp %0, %1, %2" SS_QP(0)
            : "+v"(g[0]) : "v"(Cq), "v"(dy));
}

// The read-out of Eq. 2b for a lane's SPL states: y = sum_k C_k h[k], Cq holding C like Bq above.
template <int SPL>
__device__ __forceinline__ void readout_step_dpp(float& y, float Cq, const float (&h)[STATES_PER_LANE])
{
    if constexpr (SPL == 4)
        asm("s_nop 1\n\t"
            "v_mul_f32_dpp %0, %1, %2" SS_QP(0) "\n\t"
            "v_fmac_f32_dpp %0, %1, %3" SS_QP(1) "\n\t"
            "v_fmac_f32_dpp %0, %1, %4" SS_QP(2) "\n\t"
            "v_fmac_f32_dpp %0, %1, %5" SS_QP(3)
            : "=&v"(y) : "v"(Cq), "v"(h[0]), "v"(h[1]), "v"(h[2]), "v"(h[3]));
    else if constexpr (SPL == 2)
        asm("s_nop 1\n\t"
            "v_mul_f32_dpp %0, %1, %2" SS_QP(0) "\n\t"
            "v_fmac_f32_dpp %0, %1, %3" SS_QP(1)
            : "=&v"(y) : "v"(Cq), "v"(h[0]), "v"(h[1]));
    else
        asm("s_nop 1\n\t"
            "v_mul_f32_dpp %0, %1, %2" SS_QP(0)
            : "=&v"(y) : "v"(Cq), "v"(h[0]));
}
#undef SS_QP

}  // namespace ss
