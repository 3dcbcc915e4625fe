// Diagnostic, not part of the method: ONE 32 x 32 x 64 product on the matrix instruction of the named format, operands
// and scales exactly as the caller gives them, so that a test can establish what the instruction does with hand-built
// blocks (which products of a block survive its internal accumulation).  The fused forward's choice of how MXFP8 tiles
// form Q K^T (decoded to bf16 and multiplied on the bf16 MFMA, Alg. 1 line 7 notwithstanding) rests on that evidence.
#include "dma_device.hpp"
#include "dma_internal.hpp"

namespace dma {

// a, b: row-major [32][64] elements along k (E4M3: one byte each; E2M1: two per byte, even k in the low nibble; bf16:
// two bytes each); sa, sb: [32][2] E8M0 bytes, one per row and 32-element block (ignored for bf16).
// out[i][j] = sum_k a[i][k] * b[j][k], float32 [32][32].
template <int FMT>
__global__ void __launch_bounds__(64)
diag_mfma_kernel(const uint8_t* __restrict__ a, const uint8_t* __restrict__ b, const uint8_t* __restrict__ sa,
                 const uint8_t* __restrict__ sb, float* __restrict__ out)
{
    const int lane = threadIdx.x, r = lane & 31, g = lane >> 5;
    v16f acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    if constexpr (FMT == FMT_E2M1) {
        // lane (r, g): the 32 consecutive k of block g of row r (16 bytes), and that block's scale
        const v4i av = *(const v4i*)(a + r * 32 + 16 * g), bv = *(const v4i*)(b + r * 32 + 16 * g);
        const v8i a8 = {av[0], av[1], av[2], av[3], 0, 0, 0, 0}, b8 = {bv[0], bv[1], bv[2], bv[3], 0, 0, 0, 0};
        acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, acc, 4, 4, 0, (int)sa[r * 2 + g], 0, (int)sb[r * 2 + g]);
    } else if constexpr (FMT == FMT_E4M3) {
        // lane (r, g): VGPR 0-3 = k 16 g + [0, 16), VGPR 4-7 = k 32 + 16 g + [0, 16); its scale byte is block g's
        const v4i a0 = *(const v4i*)(a + r * 64 + 16 * g), a1 = *(const v4i*)(a + r * 64 + 32 + 16 * g);
        const v4i b0 = *(const v4i*)(b + r * 64 + 16 * g), b1 = *(const v4i*)(b + r * 64 + 32 + 16 * g);
        const v8i a8 = {a0[0], a0[1], a0[2], a0[3], a1[0], a1[1], a1[2], a1[3]};
        const v8i b8 = {b0[0], b0[1], b0[2], b0[3], b1[0], b1[1], b1[2], b1[3]};
        acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, acc, 0, 0, 0, (int)sa[r * 2 + g], 0, (int)sb[r * 2 + g]);
    } else {
        // four 32 x 32 x 16 steps; lane (r, g): k = 16 step + 8 g + [0, 8)
#pragma unroll
        for (int step = 0; step < 4; ++step) {
            const v4i av = *(const v4i*)(a + (r * 64 + 16 * step + 8 * g) * 2), bv = *(const v4i*)(b + (r * 64 + 16 * step + 8 * g) * 2);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, av), __builtin_bit_cast(v8bf, bv), acc, 0, 0, 0);
        }
    }
    // accumulator: lane holds column j = r of out; VGPR t holds row i = 8 (t / 4) + 4 g + t % 4
#pragma unroll
    for (int t = 0; t < 16; ++t) out[(8 * (t / 4) + 4 * g + t % 4) * 32 + r] = acc[t];
}

// Pure instruction streams side by side on one SIMD.  One workgroup per CU; the waves of slot s (waves 4 s .. 4 s + 3, one
// per SIMD) issue stream kind[s] back to back until `ticks` of the 100 MHz wall clock have passed and add the number of
// instructions they issued to counts[s].  Every stream is a rotation over independent registers, so only the issue rate
// and the pipes limit it.  Every wave leaves its loop when the clock says so: the grid always drains.
struct PipeKinds { int k[3]; };

template <typename F>
DMA_DEV unsigned long long run_stream(long long t_end, int per_round, F&& round)
{
    unsigned long long n = 0;
    do {
        round();
        n += per_round;
    } while (wall_clock64() < t_end);
    return n;
}

__global__ void __launch_bounds__(768)
diag_pipes_kernel(PipeKinds kinds, long long ticks, unsigned long long* __restrict__ counts)
{
    const int slot = __builtin_amdgcn_readfirstlane(threadIdx.x >> 8);
    const int kind = kinds.k[slot];
    const long long t_end = wall_clock64() + ticks;
    unsigned long long n = 0;
    float sink = 0.f;
    if (kind >= 1 && kind <= 3) {
        // four accumulators in rotation, 32 instructions per look at the clock
        v16f c[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) c[i] = v16f{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        const int seed = 0x22222222 + (int)(threadIdx.x & 1);
        const v8i w8 = {seed, seed, seed, seed, seed, seed, seed, seed}, w4 = {seed, seed, seed, seed, 0, 0, 0, 0};
        const v4i h = {0x3f803f80, 0x3f803f80, 0x3f803f80, 0x3f803f80};
        if (kind == 1)
            n = run_stream(t_end, 32, [&] {
#pragma unroll
                for (int r = 0; r < 32; ++r)
                    c[r & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, h), __builtin_bit_cast(v8bf, h), c[r & 3], 0, 0, 0);
            });
        else if (kind == 2)
            n = run_stream(t_end, 32, [&] {
#pragma unroll
                for (int r = 0; r < 32; ++r) c[r & 3] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(w4, w4, c[r & 3], 4, 4, 0, 127, 0, 127);
            });
        else
            n = run_stream(t_end, 32, [&] {
#pragma unroll
                for (int r = 0; r < 32; ++r) c[r & 3] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(w8, w8, c[r & 3], 0, 0, 0, 127, 0, 127);
            });
        sink = c[0][0] + c[1][1] + c[2][2] + c[3][3];
    } else if (kind >= 4 && kind <= 6) {
        // sixteen registers in rotation, 128 instructions per look at the clock
        float x[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) x[i] = 0.001f * (float)(threadIdx.x + i + 1);
        const float mul = 0.999f, add = 0.0001f;
        if (kind == 4)
            n = run_stream(t_end, 128, [&] {
#pragma unroll
                for (int r = 0; r < 128; ++r) asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(x[r & 15]) : "v"(mul), "v"(add));
            });
        else if (kind == 5)
            n = run_stream(t_end, 128, [&] {
#pragma unroll
                for (int r = 0; r < 128; ++r) asm volatile("v_exp_f32 %0, %0" : "+v"(x[r & 15]));
            });
        else
            n = run_stream(t_end, 128, [&] {
#pragma unroll
                for (int r = 0; r < 128; ++r) asm volatile("v_cvt_pk_bf16_f32 %0, %0, %1" : "+v"(x[r & 15]) : "v"(mul));
            });
#pragma unroll
        for (int i = 0; i < 16; ++i) sink += x[i];
    }
    if (sink == 12345.678f) n += 1;                  // keeps the streams alive; never true in practice, and harmless
    if ((threadIdx.x & 63) == 0 && n) atomicAdd(&counts[slot], n);
}

int launch_diag_pipes(const int* kinds, int n_slots, long long ticks, unsigned long long* counts, hipStream_t stream)
{
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        return DMA_ERR_HIP_;
    PipeKinds pk = {{0, 0, 0}};
    for (int s = 0; s < n_slots; ++s) pk.k[s] = kinds[s];
    return launch(diag_pipes_kernel, dim3(cus), dim3(256 * n_slots), stream, pk, ticks, counts);
}

int launch_diag_mfma(const void* a, const void* b, const void* sa, const void* sb, int fmt, float* out, hipStream_t stream)
{
    const uint8_t *pa = (const uint8_t*)a, *pb = (const uint8_t*)b, *psa = (const uint8_t*)sa, *psb = (const uint8_t*)sb;
    if (fmt == FMT_E2M1) return launch(diag_mfma_kernel<FMT_E2M1>, dim3(1), dim3(64), stream, pa, pb, psa, psb, out);
    if (fmt == FMT_E4M3) return launch(diag_mfma_kernel<FMT_E4M3>, dim3(1), dim3(64), stream, pa, pb, psa, psb, out);
    if (fmt == FMT_BF16) return launch(diag_mfma_kernel<FMT_BF16>, dim3(1), dim3(64), stream, pa, pb, psa, psb, out);
    return DMA_ERR_UNSUPPORTED_;
}

}  // namespace dma
