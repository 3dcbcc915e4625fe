// Declarations shared by the translation units of the library (host side).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <tuple>
#include <utility>

namespace dma {

// Mirror of the public return codes (the public header is included only by dma_api.hip).
constexpr int DMA_OK_ = 0;
constexpr int DMA_ERR_INVALID_ARG_ = -1;
constexpr int DMA_ERR_UNSUPPORTED_ = -2;
constexpr int DMA_ERR_HIP_ = -3;

// Launch `kernel` and report what THIS launch returned: DMA_OK_ or DMA_ERR_HIP_.  (hipGetLastError() after a <<<>>> launch
// would also report, and clear, an error some earlier, unrelated HIP call of the caller's thread left behind.)
template <typename... P, size_t... I>
inline hipError_t launch_impl(void (*kernel)(P...), dim3 grid, dim3 block, hipStream_t stream, std::tuple<P...>& vals,
                              std::index_sequence<I...>)
{
    void* ptrs[] = {static_cast<void*>(&std::get<I>(vals))...};
    return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, 0, stream);
}
template <typename... P, typename... A>
inline int launch(void (*kernel)(P...), dim3 grid, dim3 block, hipStream_t stream, A... args)
{
    static_assert(sizeof...(P) == sizeof...(A), "one argument per kernel parameter");
    std::tuple<P...> vals{static_cast<P>(args)...};
    return launch_impl(kernel, grid, block, stream, vals, std::index_sequence_for<P...>{}) == hipSuccess ? DMA_OK_ : DMA_ERR_HIP_;
}

// mode: 1 = E4M3 only (c8/s8), 2 = E2M1 only (c4/s4), 3 = both, 4 = E5M2 only (c8/s8).
// token_scales: NULL, or [rows] floats receiving the per-token scale of Alg. 2 Step 2 (then applied; modes 1, 2, 4).
int launch_mx_quantize(const void* x, int64_t rows, int D, int mode, int is_query, void* c4, void* s4,
                       void* c8, void* s8, float* token_scales, hipStream_t stream);

int launch_diag_copy(const void* src, void* dst, int64_t bytes, hipStream_t stream);

// One 32 x 32 x 64 product on the matrix instruction of format fmt (product-path id of dma_device.hpp: 0, 1 or 2).
int launch_diag_mfma(const void* a, const void* b, const void* sa, const void* sb, int fmt, float* out, hipStream_t stream);

// Instruction streams of kinds[0 .. n_slots) (1 <= n_slots <= 3) side by side on every SIMD for `ticks` of the 100 MHz clock.
int launch_diag_pipes(const int* kinds, int n_slots, long long ticks, unsigned long long* counts, hipStream_t stream);

// Group maxima for Alg. 2 Step 2 (granularity 1 = row, 2 = block of block_rows rows per [S, D] matrix, 3 = everything).
int launch_group_amax(const void* x, int64_t n_mat, int64_t S, int D, int is_query, int granularity, int64_t block_rows,
                      float* amax, hipStream_t stream);

struct AttnArgs {
    const void* q;
    const void* k;
    const void* v;
    float* out;
    int B, Hq, Hkv, S, D;
    int tile;
    int band;
    int sink;        // leading key tiles in the high format
    int causal;
    int per_token;   // Alg. 2 Step 2 on queries and keys
    const float* q_amax;   // with per_token: group maxima per query row [B, Hq, S] instead of the row's own (or null)
    const float* k_amax;   // ... per key row [B, Hkv, S]
    int pv_mx;       // P V in MXFP8-E4M3 with blocks of 32 keys instead of 16-bit
    int hi_fmt, lo_fmt;
};

int launch_attn_fwd(const AttnArgs& a, hipStream_t stream);

}  // namespace dma
