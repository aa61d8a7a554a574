// Ceilings of one MI355X for the selective-scan kernels: what the vector ALU, the
// transcendental unit, the matrix pipe used as a multiply-add engine, and the HBM streams
// deliver when nothing else is in the way.  Stand-alone program; prints one line per test.
//
//   ss_ceilings [reps]
//
// Every arithmetic kernel runs `waves_per_simd` waves on every SIMD of the chip (256 CUs x 4
// SIMDs) and issues a fixed number of instructions per wave, so that
//   instructions per wave x waves per SIMD / elapsed  =  wave-instructions per SIMD per second,
// and with the issue cost known (4 cycles for a full-rate wave64 VALU instruction) the
// sustained shader clock follows from the fma test.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <vector>

#define CHECK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "%s:%d %s\n", __FILE__, __LINE__, hipGetErrorString(e_)); exit(1); } } while (0)

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr int ITERS = 32768;     // loop trips per wave
constexpr int CH = 8;            // independent chains per lane

enum Mode { FMA = 0, EXP, MIX_FWD, MIX_BWD, MFMA, MFMA_FMA, SPLIT_FMA_EXP, SPLIT_FMA_MFMA, FMA_HALF, EXP_HALF, MFMA_HALF, EXP_FMA4, EXP_FMA2 };

// one loop trip: FMA: CH fma; EXP: CH exp2; MIX_FWD: 4 x (4 fma-class + 1 exp), the forward
// recurrence's mix; MIX_BWD: 4 x (12 + 1); MFMA: 4 independent 4x4x1 fp32 MFMAs (4 multiply-adds
// per lane each); MFMA_FMA: 4 x (1 MFMA + 4 fma) in one wave, all chains independent; EXP_FMA4 / EXP_FMA2:
// 2 x (1 exp + 4 or 2 fma), independent chains.
template <int MODE>
__device__ __forceinline__ void trip(float (&x)[CH], f32x4 (&m)[4], float a, float b)
{
    if constexpr (MODE == FMA || MODE == FMA_HALF) {
#pragma unroll
        for (int i = 0; i < CH; ++i) x[i] = __builtin_fmaf(x[i], a, b);
    } else if constexpr (MODE == EXP || MODE == EXP_HALF) {
#pragma unroll
        for (int i = 0; i < CH; ++i) x[i] = __builtin_amdgcn_exp2f(x[i]);
    } else if constexpr (MODE == MIX_FWD) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float e = __builtin_amdgcn_exp2f(x[i] * a);
            const float bu = x[4 + i] * b;
            x[i] = __builtin_fmaf(e, x[i], bu);
            x[4 + i] = __builtin_fmaf(b, x[i], x[4 + i]);
        }
    } else if constexpr (MODE == MIX_BWD) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float e = __builtin_amdgcn_exp2f(x[i] * a);
            float p = x[4 + i] * b;
#pragma unroll
            for (int k = 0; k < 5; ++k) { p = __builtin_fmaf(p, a, e); x[i] = __builtin_fmaf(x[i], b, p); }
            x[4 + i] = __builtin_fmaf(e, p, x[4 + i]);
        }
    } else if constexpr (MODE == MFMA || MODE == MFMA_HALF) {
#pragma unroll
        for (int i = 0; i < 4; ++i) m[i] = __builtin_amdgcn_mfma_f32_4x4x1f32(a, b, m[i], 0, 0, 0);
    } else if constexpr (MODE == MFMA_FMA) {   // exact sequences, pinned with inline assembly
#pragma unroll
        for (int i = 0; i < 4; ++i)
            asm volatile("v_mfma_f32_4x4x1_16b_f32 %0, %5, %6, %0\n\t"
                         "v_fma_f32 %1, %5, %1, %6\n\tv_fma_f32 %2, %5, %2, %6\n\t"
                         "v_fma_f32 %3, %5, %3, %6\n\tv_fma_f32 %4, %5, %4, %6"
                         : "+v"(m[i]), "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]) : "v"(a), "v"(b));
    } else if constexpr (MODE == EXP_FMA4) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
            asm volatile("v_exp_f32 %0, %0\n\t"
                         "v_fma_f32 %1, %5, %1, %6\n\tv_fma_f32 %2, %5, %2, %6\n\t"
                         "v_fma_f32 %3, %5, %3, %6\n\tv_fma_f32 %4, %5, %4, %6"
                         : "+v"(x[i]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]), "+v"(x[5]) : "v"(a), "v"(b));
    } else if constexpr (MODE == EXP_FMA2) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
            asm volatile("v_exp_f32 %0, %0\n\t"
                         "v_fma_f32 %1, %3, %1, %4\n\tv_fma_f32 %2, %3, %2, %4"
                         : "+v"(x[i]), "+v"(x[2 + 2 * i]), "+v"(x[3 + 2 * i]) : "v"(a), "v"(b));
    }
}

// SPLIT_*: the two waves that share a SIMD (w and w + 4 of an 8-wave workgroup) run different
// instruction kinds: if the units overlap, the launch takes as long as the slower half alone.
// *_HALF: only waves 0..3 work (the other half of the split, alone).
template <int MODE>
__global__ void __launch_bounds__(512) alu_kernel(float* out, float a, float b, int iters)
{
    float x[CH];
    f32x4 m[4];
#pragma unroll
    for (int i = 0; i < CH; ++i) x[i] = a * (float)(threadIdx.x + i);
#pragma unroll
    for (int i = 0; i < 4; ++i) m[i] = f32x4{a, b, a, b};
    const int w = threadIdx.x >> 6;
    if constexpr (MODE == SPLIT_FMA_EXP) {
        if (w < 4) { for (int it = 0; it < iters; it += 8) _Pragma("unroll") for (int r = 0; r < 8; ++r) trip<FMA>(x, m, a, b); }
        else       { for (int it = 0; it < iters; it += 8) _Pragma("unroll") for (int r = 0; r < 8; ++r) trip<EXP>(x, m, a, b); }
    } else if constexpr (MODE == SPLIT_FMA_MFMA) {
        if (w < 4) { for (int it = 0; it < iters; it += 8) _Pragma("unroll") for (int r = 0; r < 8; ++r) trip<FMA>(x, m, a, b); }
        else       { for (int it = 0; it < iters; it += 8) _Pragma("unroll") for (int r = 0; r < 8; ++r) trip<MFMA>(x, m, a, b); }
    } else if constexpr (MODE == FMA_HALF || MODE == EXP_HALF || MODE == MFMA_HALF) {
        if (w < 4) { for (int it = 0; it < iters; it += 8) _Pragma("unroll") for (int r = 0; r < 8; ++r) trip<MODE>(x, m, a, b); }
    } else {
        for (int it = 0; it < iters; it += 8) _Pragma("unroll") for (int r = 0; r < 8; ++r) trip<MODE>(x, m, a, b);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < CH; ++i) s += x[i];
#pragma unroll
    for (int i = 0; i < 4; ++i) s += m[i][0] + m[i][1] + m[i][2] + m[i][3];
    if (s == 12345.678f) out[threadIdx.x] = s;   // never true; keeps the arithmetic alive
}

// Operand layout of the 4x4x1 fp32 MFMA (16 blocks of four lanes): the scan kernels rely on
//   out[i][lane] = a[(lane & ~3) + i] * b[lane] + c[i][lane],
// i.e. within every group of four lanes, lane i's `a` scales output register i of all four lanes.
__global__ void mfma_layout_kernel(const float* a, const float* b, const float* c, float* out)
{
    const int l = threadIdx.x;
    f32x4 acc = {c[l], c[64 + l], c[128 + l], c[192 + l]};
    acc = __builtin_amdgcn_mfma_f32_4x4x1f32(a[l], b[l], acc, 0, 0, 0);
    for (int i = 0; i < 4; ++i) out[64 * i + l] = acc[i];
}
static void check_mfma_layout()
{
    float ha[64], hb[64], hc[256], ho[256], *da, *db, *dc, *dout;
    for (int l = 0; l < 64; ++l) { ha[l] = 1.0f + 0.25f * l; hb[l] = 3.0f - 0.5f * l; }
    for (int i = 0; i < 256; ++i) hc[i] = 0.125f * i;
    CHECK(hipMalloc(&da, sizeof ha)); CHECK(hipMalloc(&db, sizeof hb)); CHECK(hipMalloc(&dc, sizeof hc)); CHECK(hipMalloc(&dout, sizeof ho));
    CHECK(hipMemcpy(da, ha, sizeof ha, hipMemcpyHostToDevice));
    CHECK(hipMemcpy(db, hb, sizeof hb, hipMemcpyHostToDevice));
    CHECK(hipMemcpy(dc, hc, sizeof hc, hipMemcpyHostToDevice));
    mfma_layout_kernel<<<dim3(1), dim3(64), 0, 0>>>(da, db, dc, dout);
    CHECK(hipMemcpy(ho, dout, sizeof ho, hipMemcpyDeviceToHost));
    int bad = 0;
    for (int i = 0; i < 4; ++i)
        for (int l = 0; l < 64; ++l)
            if (ho[64 * i + l] != ha[(l & ~3) + i] * hb[l] + hc[64 * i + l]) ++bad;
    printf("mfma_f32_4x4x1 layout out[i][l] = a[(l&~3)+i] * b[l] + c[i][l]: %s (%d mismatches)\n", bad ? "FAIL" : "PASS", bad);
    CHECK(hipFree(da)); CHECK(hipFree(db)); CHECK(hipFree(dc)); CHECK(hipFree(dout));
}

// HBM streams over rows of 16-byte pieces: read (sum kept alive), write, copy
__global__ void __launch_bounds__(256) stream_read(const u32x4* __restrict__ src, long n, uint32_t* out)
{
    uint32_t acc = 0;
    for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (long)gridDim.x * blockDim.x) {
        const u32x4 v = __builtin_nontemporal_load(src + i);
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    if (acc == 0x12345678u) out[0] = acc;
}
__global__ void __launch_bounds__(256) stream_write(u32x4* __restrict__ dst, long n, uint32_t v)
{
    for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (long)gridDim.x * blockDim.x)
        dst[i] = u32x4{v, v, v, v};
}
__global__ void __launch_bounds__(256) stream_copy(const u32x4* __restrict__ src, u32x4* __restrict__ dst, long n)
{
    for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (long)gridDim.x * blockDim.x)
        dst[i] = __builtin_nontemporal_load(src + i);
}

template <typename F>
static double time_ms(F launch, int reps)
{
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    launch();
    CHECK(hipDeviceSynchronize());
    double best = 1e30;
    for (int r = 0; r < reps; ++r) {
        CHECK(hipEventRecord(e0, 0));
        launch();
        CHECK(hipEventRecord(e1, 0));
        CHECK(hipEventSynchronize(e1));
        float ms = 0.f;
        CHECK(hipEventElapsedTime(&ms, e0, e1));
        if (ms < best) best = ms;
    }
    CHECK(hipEventDestroy(e0));
    CHECK(hipEventDestroy(e1));
    return best;
}

// The scan kernels' access pattern without their arithmetic.  A workgroup of 256 threads owns 64
// rows of row_bytes each (consecutive rows row_bytes apart, as in a (B, D, L) tensor) and walks along
// them; per trip it reads PIECE bytes of every row from each of NIN tensors and writes PIECE bytes of
// every row to each of NOUT tensors, VB bytes per thread and request, with the reads requested DEPTH
// trips ahead.  PIECE = 64, VB = 16 is the forward scan (a 32-step chunk of bf16), PIECE = 32, VB = 8
// the backward scan (a 16-step block); larger pieces show what longer contiguous runs would buy.
template <int VB> struct piece_t;
template <> struct piece_t<16> { typedef u32x4 type; };
template <> struct piece_t<8> { typedef uint32_t __attribute__((ext_vector_type(2))) type; };
template <int PIECE, int VB, int NIN, int NOUT, int DEPTH>
__global__ void __launch_bounds__(256, 2) tile_stream(const char* __restrict__ src, char* __restrict__ dst, long tensor_bytes,
                                                       int row_bytes, int ntrips)
{
    typedef typename piece_t<VB>::type V;
    constexpr int TPR = PIECE / VB;                      // threads per row
    constexpr int RPP = 256 / TPR;                       // rows per pass
    constexpr int PASSES = 64 / RPP > 0 ? 64 / RPP : 1;  // passes over the 64 rows (threads past row 63 idle)
    const int tid = threadIdx.x;
    const int r = tid / TPR, q = tid % TPR;
    if (r >= 64) return;
    const long base = (long)blockIdx.x * 64 * row_bytes + (long)r * row_bytes + q * VB;
    V buf[DEPTH][PASSES][NIN];
    uint32_t acc = 0;   // keeps the reads alive when nothing is written
    auto issue = [&](int trip, int slot) {
        const int tr = trip < ntrips ? trip : ntrips - 1;
#pragma unroll
        for (int p = 0; p < PASSES; ++p)
#pragma unroll
            for (int i = 0; i < NIN; ++i)
                buf[slot][p][i] = __builtin_nontemporal_load(reinterpret_cast<const V*>(src + i * tensor_bytes + base + (long)p * RPP * row_bytes + (long)tr * PIECE));
    };
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) issue(d, d);
    for (int trip = 0; trip < ntrips; trip += DEPTH) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
#pragma unroll
            for (int p = 0; p < PASSES; ++p) {
                V v = buf[d][p][0];
#pragma unroll
                for (int i = 1; i < NIN; ++i) v ^= buf[d][p][i];
                acc ^= v.x;
#pragma unroll
                for (int o = 0; o < NOUT; ++o)
                    *reinterpret_cast<V*>(dst + o * tensor_bytes + base + (long)p * RPP * row_bytes + (long)(trip + d) * PIECE) = v + (uint32_t)o;
            }
            issue(trip + d + DEPTH, d);
        }
    }
    if (acc == 0x12345678u) *reinterpret_cast<uint32_t*>(dst) = acc;
}

template <int PIECE, int VB, int NIN, int NOUT, int DEPTH>
static void run_tile(const char* what, const char* src, char* dst, int reps)
{
    const int rows = 8 * 4096, row_bytes = 2048 * 2;   // batch 8, 4096 channels, 2048 steps of bf16
    const long tensor_bytes = (long)rows * row_bytes;
    const int ntrips = row_bytes / PIECE;              // a multiple of DEPTH
    const double ms = time_ms([&] { tile_stream<PIECE, VB, NIN, NOUT, DEPTH><<<dim3(rows / 64), dim3(256), 0, 0>>>(src, dst, tensor_bytes, row_bytes, ntrips); }, reps);
    const double bytes = (double)(NIN + NOUT) * tensor_bytes;
    printf("row tiles, %3d-byte pieces (%2d B/thread), %d in + %d out, %d trips ahead: %7.3f ms  %7.1f GB/s   [%s]\n", PIECE, VB, NIN, NOUT, DEPTH, ms,
           bytes / (ms * 1e6), what);
}

// The same, with the scan kernels' thread mapping kept (thread = row tid / 4, quarter tid % 4 of a
// 4 * VB-byte piece) and a trip covering SPLIT such pieces of every row, requested and written back
// to back: what grouping the traffic of SPLIT chunks buys without changing who owns which element.
template <int VB, int SPLIT, int NIN, int NOUT, int DEPTH>
__global__ void __launch_bounds__(256, 2) tile_stream_split(const char* __restrict__ src, char* __restrict__ dst, long tensor_bytes,
                                                             int row_bytes, int ntrips)
{
    typedef typename piece_t<VB>::type V;
    constexpr int SUB = 4 * VB, PIECE = SUB * SPLIT;
    const int tid = threadIdx.x;
    const int r = tid >> 2, q = tid & 3;
    const long base = (long)blockIdx.x * 64 * row_bytes + (long)r * row_bytes + q * VB;
    V buf[DEPTH][SPLIT][NIN];
    uint32_t acc = 0;
    auto issue = [&](int trip, int slot) {
        const int tr = trip < ntrips ? trip : ntrips - 1;
#pragma unroll
        for (int i = 0; i < NIN; ++i)
#pragma unroll
            for (int j = 0; j < SPLIT; ++j)
                buf[slot][j][i] = __builtin_nontemporal_load(reinterpret_cast<const V*>(src + i * tensor_bytes + base + (long)tr * PIECE + j * SUB));
    };
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) issue(d, d);
    for (int trip = 0; trip < ntrips; trip += DEPTH) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            V v[SPLIT];
#pragma unroll
            for (int j = 0; j < SPLIT; ++j) {
                v[j] = buf[d][j][0];
#pragma unroll
                for (int i = 1; i < NIN; ++i) v[j] ^= buf[d][j][i];
                acc ^= v[j].x;
            }
#pragma unroll
            for (int o = 0; o < NOUT; ++o)
#pragma unroll
                for (int j = 0; j < SPLIT; ++j)
                    *reinterpret_cast<V*>(dst + o * tensor_bytes + base + (long)(trip + d) * PIECE + j * SUB) = v[j] + (uint32_t)o;
            issue(trip + d + DEPTH, d);
        }
    }
    if (acc == 0x12345678u) *reinterpret_cast<uint32_t*>(dst) = acc;
}

template <int VB, int SPLIT, int NIN, int NOUT, int DEPTH>
static void run_tile_split(const char* what, const char* src, char* dst, int reps)
{
    const int rows = 8 * 4096, row_bytes = 2048 * 2;
    const long tensor_bytes = (long)rows * row_bytes;
    const int ntrips = row_bytes / (4 * VB * SPLIT);
    const double ms = time_ms([&] { tile_stream_split<VB, SPLIT, NIN, NOUT, DEPTH><<<dim3(rows / 64), dim3(256), 0, 0>>>(src, dst, tensor_bytes, row_bytes, ntrips); }, reps);
    const double bytes = (double)(NIN + NOUT) * tensor_bytes;
    printf("row tiles, %d x %2d-byte pieces back to back, %d in + %d out, %d trips ahead: %7.3f ms  %7.1f GB/s   [%s]\n", SPLIT, 4 * VB, NIN, NOUT, DEPTH, ms,
           bytes / (ms * 1e6), what);
}

template <int MODE>
static void run_alu(const char* name, double instr_per_trip_per_wave, const char* what, float* out, int reps)
{
    // 256 CUs x 1 workgroup of 8 waves = 2 waves per SIMD
    const double ms = time_ms([&] { alu_kernel<MODE><<<dim3(256), dim3(512), 0, 0>>>(out, 1.0000001f, 1e-9f, ITERS); }, reps);
    // wave-instructions per SIMD: 2 waves (or 1 in the *_HALF and half of each in SPLIT modes; the caller's
    // count is per SIMD) x trips x instructions
    const double per_simd = instr_per_trip_per_wave * ITERS;
    printf("%-16s %8.3f ms  %9.1f wave-instr/us/SIMD  => %6.2f cycles/instr at 2.4 GHz   [%s]\n", name, ms,
           per_simd / (ms * 1e3), ms * 1e-3 * 2.4e9 / per_simd, what);
}

int main(int argc, char** argv)
{
    const int reps = argc > 1 ? atoi(argv[1]) : 5;
    hipDeviceProp_t prop;
    CHECK(hipGetDeviceProperties(&prop, 0));
    printf("device: %s, %d CUs, clock %d kHz, memory clock %d kHz\n", prop.gcnArchName, prop.multiProcessorCount,
           prop.clockRate, prop.memoryClockRate);
    check_mfma_layout();
    float* out;
    CHECK(hipMalloc(&out, 4096));
    // counts are wave-instructions issued on ONE SIMD per loop trip (2 resident waves unless noted)
    run_alu<FMA>("fma", 2.0 * CH, "v_fma_f32, 2 waves/SIMD", out, reps);
    run_alu<FMA_HALF>("fma_1wave", 1.0 * CH, "v_fma_f32, 1 wave/SIMD", out, reps);
    run_alu<EXP>("exp", 2.0 * CH, "v_exp_f32, 2 waves/SIMD", out, reps);
    run_alu<EXP_HALF>("exp_1wave", 1.0 * CH, "v_exp_f32, 1 wave/SIMD", out, reps);
    run_alu<MIX_FWD>("mix_fwd", 2.0 * 4 * 5, "4 x (mul, exp, mul, fma, fma), counted as 5", out, reps);
    run_alu<MIX_BWD>("mix_bwd", 2.0 * 4 * 14, "4 x (exp + 13 fma-class), counted as 14", out, reps);
    run_alu<MFMA>("mfma4x4x1", 2.0 * 4, "v_mfma_f32_4x4x1_16b_f32, 2 waves/SIMD", out, reps);
    run_alu<MFMA_HALF>("mfma_1wave", 1.0 * 4, "the same, 1 wave/SIMD", out, reps);
    run_alu<MFMA_FMA>("mfma+4fma", 2.0 * 20, "4 x (1 mfma + 4 fma) in one wave, independent, counted as 20", out, reps);
    run_alu<EXP_FMA4>("exp+4fma", 2.0 * 10, "2 x (1 exp + 4 fma), independent, counted as 10", out, reps);
    run_alu<EXP_FMA2>("exp+2fma", 2.0 * 6, "2 x (1 exp + 2 fma), independent, counted as 6", out, reps);
    run_alu<SPLIT_FMA_EXP>("fma|exp", 2.0 * CH, "one wave fma, the other exp, same SIMD", out, reps);
    run_alu<SPLIT_FMA_MFMA>("fma|mfma", 1.0 * CH + 4, "one wave 8 fma, the other 4 mfma per trip", out, reps);

    const long bytes = 1L << 30;
    const long n = bytes / 16;
    u32x4 *src, *dst;
    CHECK(hipMalloc(&src, bytes));
    CHECK(hipMalloc(&dst, bytes));
    CHECK(hipMemset(src, 1, bytes));
    CHECK(hipMemset(dst, 2, bytes));
    for (int blocks : {1024, 2048, 4096, 8192}) {
        const double r = time_ms([&] { stream_read<<<dim3(blocks), dim3(256), 0, 0>>>(src, n, (uint32_t*)out); }, reps);
        const double w = time_ms([&] { stream_write<<<dim3(blocks), dim3(256), 0, 0>>>(dst, n, 7u); }, reps);
        const double c = time_ms([&] { stream_copy<<<dim3(blocks), dim3(256), 0, 0>>>(src, dst, n); }, reps);
        printf("stream 1 GiB, %5d workgroups: read %7.1f GB/s   write %7.1f GB/s   copy %7.1f GB/s (read+write)\n", blocks,
               bytes / (r * 1e6), bytes / (w * 1e6), 2.0 * bytes / (c * 1e6));
    }
    // (B, D, L) = (8, 4096, 2048) bf16 tensors: 7 inputs + 4 outputs of 128 MiB fit the two 1 GiB buffers
    run_tile<64, 16, 3, 4, 2>("forward scan: u, delta, z in; out, y and 4 bytes/step of checkpoints out", (const char*)src, (char*)dst, reps);
    run_tile<64, 16, 3, 2, 2>("forward scan without the checkpoints", (const char*)src, (char*)dst, reps);
    run_tile<128, 16, 3, 4, 2>("the same bytes in 128-byte pieces", (const char*)src, (char*)dst, reps);
    run_tile<256, 16, 3, 4, 2>("the same bytes in 256-byte pieces", (const char*)src, (char*)dst, reps);
    run_tile<64, 16, 3, 4, 4>("forward scan, four trips ahead", (const char*)src, (char*)dst, reps);
    run_tile<32, 8, 7, 3, 2>("backward scan: u, delta, z, dout, y + 4 bytes/step of checkpoints in; du, ddelta, dz out", (const char*)src, (char*)dst, reps);
    run_tile<32, 8, 7, 3, 4>("backward scan, four trips ahead", (const char*)src, (char*)dst, reps);
    run_tile<64, 16, 7, 3, 2>("the same bytes in 64-byte pieces", (const char*)src, (char*)dst, reps);
    run_tile<128, 16, 7, 3, 2>("the same bytes in 128-byte pieces", (const char*)src, (char*)dst, reps);
    run_tile<64, 16, 3, 0, 2>("reads only, 64-byte pieces", (const char*)src, (char*)dst, reps);
    run_tile<64, 16, 1, 4, 2>("mostly writes, 64-byte pieces", (const char*)src, (char*)dst, reps);
    run_tile_split<16, 2, 3, 4, 2>("forward bytes, two chunks' traffic grouped", (const char*)src, (char*)dst, reps);
    run_tile_split<16, 4, 3, 4, 2>("forward bytes, four chunks' traffic grouped", (const char*)src, (char*)dst, reps);
    run_tile_split<16, 4, 3, 4, 1>("forward bytes, four chunks' traffic grouped, one trip ahead", (const char*)src, (char*)dst, reps);
    run_tile_split<8, 2, 7, 3, 2>("backward bytes, two blocks' traffic grouped", (const char*)src, (char*)dst, reps);
    run_tile_split<8, 4, 7, 3, 2>("backward bytes, four blocks' traffic grouped", (const char*)src, (char*)dst, reps);
    run_tile_split<8, 8, 7, 3, 1>("backward bytes, eight blocks' traffic grouped, one trip ahead", (const char*)src, (char*)dst, reps);
    run_tile_split<16, 2, 1, 4, 2>("mostly writes, two 64-byte pieces back to back", (const char*)src, (char*)dst, reps);
    run_tile_split<16, 4, 1, 4, 2>("mostly writes, four 64-byte pieces back to back", (const char*)src, (char*)dst, reps);
    CHECK(hipFree(src));
    CHECK(hipFree(dst));
    CHECK(hipFree(out));
    return 0;
}
