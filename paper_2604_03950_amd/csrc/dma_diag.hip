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

int launch_diag_mfma(const void* a, const void* b, const void* sa, const void* sb, int fmt, float* out, hipStream_t stream)
{
    const uint8_t *pa = (const uint8_t*)a, *pb = (const uint8_t*)b, *psa = (const uint8_t*)sa, *psb = (const uint8_t*)sb;
    if (fmt == FMT_E2M1) return launch(diag_mfma_kernel<FMT_E2M1>, dim3(1), dim3(64), stream, pa, pb, psa, psb, out);
    if (fmt == FMT_E4M3) return launch(diag_mfma_kernel<FMT_E4M3>, dim3(1), dim3(64), stream, pa, pb, psa, psb, out);
    if (fmt == FMT_BF16) return launch(diag_mfma_kernel<FMT_BF16>, dim3(1), dim3(64), stream, pa, pb, psa, psb, out);
    return DMA_ERR_UNSUPPORTED_;
}

}  // namespace dma
