// Standalone MX quantizer (paper, Alg. 2 Steps 1, 3-7; Alg. 3): one streaming pass, HBM bound.
//
// Work split: one lane converts one 16-byte chunk (8 bf16); the 4 lanes of a quad hold one MX block
// of 32 elements, so the block maximum is two DPP quad permutes.  Loads are 16 B per lane and
// contiguous across the wave; code stores are 4 B (FP4) / 8 B (FP8) per lane, contiguous; the scale
// byte is written by the first lane of each quad.
#include "dma_device.hpp"
#include "dma_internal.hpp"
#include <math.h>

namespace dma {

constexpr int QUANT_THREADS = 256;
constexpr int QUANT_UNROLL = 4;     // chunks per thread

// MODE: 1 = E4M3 only, 2 = E2M1 only, 3 = both (low copy E2M1 + high copy E4M3), 4 = E5M2 only.
// PER_TOKEN: Alg. 2 Step 2: the row (lanes_per_row = D / 8 consecutive lanes, a power of two <= 64) is multiplied by
// 2688 / rowmax before the shared scales are formed, and rowmax / 2688 goes to token_scales[row].
template <int MODE, bool IS_QUERY, bool PER_TOKEN>
__global__ void __launch_bounds__(QUANT_THREADS)
mx_quantize_kernel(const v4i* __restrict__ x, int64_t n_chunks, float c,
                   int* __restrict__ codes4, uint8_t* __restrict__ scales4,
                   v2i* __restrict__ codes8, uint8_t* __restrict__ scales8,
                   float* __restrict__ token_scales, int lanes_per_row)
{
    const int64_t base = ((int64_t)blockIdx.x * QUANT_UNROLL) * QUANT_THREADS + threadIdx.x;
    v4i w[QUANT_UNROLL];
#pragma unroll
    for (int u = 0; u < QUANT_UNROLL; ++u) {
        const int64_t ch = base + (int64_t)u * QUANT_THREADS;
        w[u] = (ch < n_chunks) ? __builtin_nontemporal_load(x + ch) : v4i{0, 0, 0, 0};
    }
#pragma unroll
    for (int u = 0; u < QUANT_UNROLL; ++u) {
        const int64_t ch = base + (int64_t)u * QUANT_THREADS;
        float v[8];
        unpack8<IS_QUERY>(w[u], c, v);
        if constexpr (PER_TOKEN) {
            // row maximum: quad, then butterfly over the remaining lanes of the row (rows never straddle a wave)
            float rmax = quad_max(amax8(v));
            for (int off = 4; off < lanes_per_row; off <<= 1) rmax = fmaxf(rmax, __shfl_xor(rmax, off, 64));
            float s_q, inv;
            token_scale(rmax, s_q, inv);
#pragma unroll
            for (int t = 0; t < 8; ++t) v[t] = __fmul_rn(v[t], inv);
            if (ch < n_chunks && (ch % lanes_per_row) == 0) token_scales[ch / lanes_per_row] = s_q;
        }
        const float amax = quad_max(amax8(v));      // every lane of the wave executes the DPP
        if (ch >= n_chunks) continue;
        const bool writes_scale = (threadIdx.x & 3) == 0;
        if (MODE & 2) {
            const int code = e8m0_code<FMT_E2M1>(amax);
            __builtin_nontemporal_store(encode8_e2m1(v, code), codes4 + ch);
            if (writes_scale) scales4[ch >> 2] = (uint8_t)code;
        }
        if (MODE & 1) {
            const int code = e8m0_code<FMT_E4M3>(amax);
            __builtin_nontemporal_store(encode8_e4m3(v, code), codes8 + ch);
            if (writes_scale) scales8[ch >> 2] = (uint8_t)code;
        }
        if (MODE & 4) {
            const int code = e8m0_code<FMT_E5M2_X>(amax);
            __builtin_nontemporal_store(encode8_e5m2(v, code), codes8 + ch);
            if (writes_scale) scales8[ch >> 2] = (uint8_t)code;
        }
    }
}

template <int MODE, bool PER_TOKEN>
static int launch_mode(const void* x, int64_t rows, int D, int is_query, void* c4, void* s4, void* c8,
                       void* s8, float* ts, hipStream_t stream)
{
    const int64_t n_chunks = rows * (int64_t)(D / 8);
    if (n_chunks == 0) return DMA_OK_;
    const int64_t per_block = (int64_t)QUANT_THREADS * QUANT_UNROLL;
    const int64_t blocks = (n_chunks + per_block - 1) / per_block;
    if (blocks > 0x7fffffffLL) return DMA_ERR_UNSUPPORTED_;
    const float c = (float)(1.4426950408889634074 / sqrt((double)D));
    const int lpr = D / 8;
    if (PER_TOKEN && (lpr > 64 || (lpr & (lpr - 1)) != 0)) return DMA_ERR_UNSUPPORTED_;
    if (is_query)
        return launch(mx_quantize_kernel<MODE, true, PER_TOKEN>, dim3((unsigned)blocks), dim3(QUANT_THREADS), stream,
                      (const v4i*)x, n_chunks, c, (int*)c4, (uint8_t*)s4, (v2i*)c8, (uint8_t*)s8, ts, lpr);
    return launch(mx_quantize_kernel<MODE, false, PER_TOKEN>, dim3((unsigned)blocks), dim3(QUANT_THREADS), stream,
                  (const v4i*)x, n_chunks, c, (int*)c4, (uint8_t*)s4, (v2i*)c8, (uint8_t*)s8, ts, lpr);
}

// Plain copy, 16 bytes per lane: the reference kernel for calibrating HBM traffic counters.
__global__ void __launch_bounds__(QUANT_THREADS)
diag_copy_kernel(const v4i* __restrict__ src, v4i* __restrict__ dst, int64_t n_chunks)
{
    const int64_t i = (int64_t)blockIdx.x * QUANT_THREADS + threadIdx.x;
    if (i < n_chunks) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

int launch_diag_copy(const void* src, void* dst, int64_t bytes, hipStream_t stream)
{
    const int64_t n_chunks = bytes / 16;
    if (n_chunks == 0) return DMA_OK_;
    const int64_t blocks = (n_chunks + QUANT_THREADS - 1) / QUANT_THREADS;
    if (blocks > 0x7fffffffLL) return DMA_ERR_UNSUPPORTED_;
    return launch(diag_copy_kernel, dim3((unsigned)blocks), dim3(QUANT_THREADS), stream, (const v4i*)src, (v4i*)dst, n_chunks);
}

// ---------------------------------------------------------------------------------------------
// Group maxima for Alg. 2 Step 2 at a coarser granularity than the row (Sec. 5.3 names per-block and per-tensor).
// First the maximum magnitude of every row (queries: after the pre-scale; the product is monotone, so it is taken of
// the row maximum), then, in place, the maximum over the block of rows or over everything.
// ---------------------------------------------------------------------------------------------
template <int LPR>                                    // lanes per row: D / 8
__global__ void __launch_bounds__(QUANT_THREADS)
row_amax_kernel(const v4i* __restrict__ x, int64_t rows, float c, int prescale, float* __restrict__ out)
{
    const int64_t t = (int64_t)blockIdx.x * QUANT_THREADS + threadIdx.x;      // one 16-byte chunk per thread
    const int64_t row = t / LPR;
    float a = 0.f;
    if (row < rows) {
        float v[8];
        unpack8<false>(x[t], 1.f, v);
        a = amax8(v);
    }
    a = group_max<LPR>(a);
    if (row < rows && t % LPR == 0) out[row] = prescale ? __fmul_rn(a, c) : a;
}

DMA_DEV float wave_max(float a)
{
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) a = fmaxf(a, __shfl_xor(a, m, 64));
    return a;
}

// One wave per (matrix, block of block_rows rows): maximum of the block, written to each of its rows.
__global__ void __launch_bounds__(64)
block_amax_kernel(float* __restrict__ amax, int64_t S, int64_t block_rows, int64_t blocks_per_matrix)
{
    const int64_t mtx = blockIdx.x / blocks_per_matrix, blk = blockIdx.x % blocks_per_matrix;
    const int64_t r0 = blk * block_rows, r1 = (r0 + block_rows < S) ? r0 + block_rows : S;
    float* p = amax + mtx * S;
    float a = 0.f;
    for (int64_t r = r0 + threadIdx.x; r < r1; r += 64) a = fmaxf(a, p[r]);
    a = wave_max(a);
    for (int64_t r = r0 + threadIdx.x; r < r1; r += 64) p[r] = a;
}

// Per-tensor maximum in three steps: block maxima over runs of TENSOR_RUN rows (block_amax_kernel), one workgroup that
// reduces the first row of every run into amax[0], and a grid that copies amax[0] to every row.
constexpr int64_t TENSOR_RUN = 1024;
__global__ void __launch_bounds__(1024)
tensor_reduce_kernel(float* __restrict__ amax, int64_t rows)
{
    __shared__ float part[16];
    float a = 0.f;
    for (int64_t r = (int64_t)threadIdx.x * TENSOR_RUN; r < rows; r += 1024 * TENSOR_RUN) a = fmaxf(a, amax[r]);
    a = wave_max(a);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = a;
    __syncthreads();
    if (threadIdx.x == 0) {
        a = part[0];
#pragma unroll
        for (int w = 1; w < 16; ++w) a = fmaxf(a, part[w]);
        amax[0] = a;
    }
}
__global__ void __launch_bounds__(QUANT_THREADS)
broadcast_first_kernel(float* __restrict__ amax, int64_t rows)
{
    const int64_t r = (int64_t)blockIdx.x * QUANT_THREADS + threadIdx.x;
    const float a = amax[0];              // row 0 is rewritten with the value it already holds
    if (r < rows) amax[r] = a;
}

// granularity: 1 = the row, 2 = blocks of block_rows rows of each [S, D] matrix, 3 = everything.  D is 64 or 128.
int launch_group_amax(const void* x, int64_t n_mat, int64_t S, int D, int is_query, int granularity, int64_t block_rows,
                      float* amax, hipStream_t stream)
{
    const int64_t rows = n_mat * S;
    const int64_t chunks = rows * (D / 8);
    const int64_t blocks = (chunks + QUANT_THREADS - 1) / QUANT_THREADS;
    if (blocks > 0x7fffffffLL) return DMA_ERR_UNSUPPORTED_;
    const float c = (float)(1.4426950408889634074 / sqrt((double)D));
    // every size check comes before the first launch: on error nothing has been enqueued
    const int64_t bpm = granularity == 2 ? (S + block_rows - 1) / block_rows : 0;
    const int64_t runs = (rows + TENSOR_RUN - 1) / TENSOR_RUN;
    if (D != 128 && D != 64) return DMA_ERR_UNSUPPORTED_;
    if ((granularity == 2 && n_mat * bpm > 0x7fffffffLL) || (granularity == 3 && runs > 0x7fffffffLL)) return DMA_ERR_UNSUPPORTED_;
    int rc = D == 128 ? launch(row_amax_kernel<16>, dim3((unsigned)blocks), dim3(QUANT_THREADS), stream, (const v4i*)x, rows, c, is_query, amax)
                      : launch(row_amax_kernel<8>, dim3((unsigned)blocks), dim3(QUANT_THREADS), stream, (const v4i*)x, rows, c, is_query, amax);
    if (rc == DMA_OK_ && granularity == 2)
        rc = launch(block_amax_kernel, dim3((unsigned)(n_mat * bpm)), dim3(64), stream, amax, S, block_rows, bpm);
    if (granularity == 3) {
        if (rc == DMA_OK_) rc = launch(block_amax_kernel, dim3((unsigned)runs), dim3(64), stream, amax, rows, TENSOR_RUN, runs);
        if (rc == DMA_OK_) rc = launch(tensor_reduce_kernel, dim3(1), dim3(1024), stream, amax, rows);
        if (rc == DMA_OK_) rc = launch(broadcast_first_kernel, dim3((unsigned)((rows + QUANT_THREADS - 1) / QUANT_THREADS)), dim3(QUANT_THREADS), stream, amax, rows);
    }
    return rc;
}

int launch_mx_quantize(const void* x, int64_t rows, int D, int mode, int is_query, void* c4, void* s4,
                       void* c8, void* s8, float* token_scales, hipStream_t stream)
{
    if (token_scales) {
        switch (mode) {
            case 1: return launch_mode<1, true>(x, rows, D, is_query, c4, s4, c8, s8, token_scales, stream);
            case 2: return launch_mode<2, true>(x, rows, D, is_query, c4, s4, c8, s8, token_scales, stream);
            case 4: return launch_mode<4, true>(x, rows, D, is_query, c4, s4, c8, s8, token_scales, stream);
        }
        return DMA_ERR_INVALID_ARG_;
    }
    switch (mode) {
        case 1: return launch_mode<1, false>(x, rows, D, is_query, c4, s4, c8, s8, nullptr, stream);
        case 2: return launch_mode<2, false>(x, rows, D, is_query, c4, s4, c8, s8, nullptr, stream);
        case 3: return launch_mode<3, false>(x, rows, D, is_query, c4, s4, c8, s8, nullptr, stream);
        case 4: return launch_mode<4, false>(x, rows, D, is_query, c4, s4, c8, s8, nullptr, stream);
    }
    return DMA_ERR_INVALID_ARG_;
}

}  // namespace dma
