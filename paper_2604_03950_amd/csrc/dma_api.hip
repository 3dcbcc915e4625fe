// C ABI entry points: argument checks and dispatch.  Every step of the path runs in the kernels.
#include "../../include/dma.h"
#include "dma_internal.hpp"

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool valid_fmt(int f) { return f == DMA_FMT_BF16 || f == DMA_FMT_MXFP8_E4M3 || f == DMA_FMT_MXFP4_E2M1 || f == DMA_FMT_MXFP8_E5M2; }

// rows == 0 is a no-op that never looks at the pointers (an empty tensor has none).
int check_quant_common(const void* x, int64_t rows, int D)
{
    if (rows < 0) return DMA_ERR_INVALID_ARG;
    if (D < 32 || D > 1024 || D % 32 != 0) return DMA_ERR_INVALID_ARG;
    if (rows == 0) return DMA_OK;
    if (!x) return DMA_ERR_INVALID_ARG;
    if (!aligned16(x)) return DMA_ERR_INVALID_ARG;
    if (rows > (int64_t)1 << 40) return DMA_ERR_UNSUPPORTED;
    return DMA_OK;
}

}  // namespace

static int quantize_one(const void* x_bf16, int64_t rows, int D, int fmt, int is_query, void* codes_u8,
                        void* scales_u8, float* token_scales, bool per_token, void* stream)
{
    int rc = check_quant_common(x_bf16, rows, D);
    if (rc != DMA_OK) return rc;
    if (fmt != DMA_FMT_MXFP8_E4M3 && fmt != DMA_FMT_MXFP4_E2M1 && fmt != DMA_FMT_MXFP8_E5M2) return DMA_ERR_INVALID_ARG;
    if (rows == 0) return DMA_OK;
    if (!codes_u8 || !scales_u8 || (per_token && !token_scales)) return DMA_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(codes_u8) & 7u) != 0) return DMA_ERR_INVALID_ARG;
    if (per_token && (reinterpret_cast<uintptr_t>(token_scales) & 3u) != 0) return DMA_ERR_INVALID_ARG;
    if (fmt == DMA_FMT_MXFP4_E2M1)
        return dma::launch_mx_quantize(x_bf16, rows, D, 2, is_query != 0, codes_u8, scales_u8, nullptr, nullptr,
                                       token_scales, (hipStream_t)stream);
    return dma::launch_mx_quantize(x_bf16, rows, D, fmt == DMA_FMT_MXFP8_E5M2 ? 4 : 1, is_query != 0, nullptr, nullptr,
                                   codes_u8, scales_u8, token_scales, (hipStream_t)stream);
}

extern "C" {

int dma_mx_quantize(const void* x_bf16, int64_t rows, int D, int fmt, int is_query, void* codes_u8,
                    void* scales_u8, void* stream)
{
    return quantize_one(x_bf16, rows, D, fmt, is_query, codes_u8, scales_u8, nullptr, false, stream);
}

int dma_mx_quantize_token(const void* x_bf16, int64_t rows, int D, int fmt, int is_query, void* codes_u8,
                          void* scales_u8, void* token_scales_f32, void* stream)
{
    return quantize_one(x_bf16, rows, D, fmt, is_query, codes_u8, scales_u8, (float*)token_scales_f32, true, stream);
}

int dma_mx_group_amax(const void* x_bf16, int64_t n_mat, int64_t S, int D, int is_query, int granularity,
                      int64_t block_rows, void* amax_f32, void* stream)
{
    if (n_mat < 0 || S < 0 || D <= 0) return DMA_ERR_INVALID_ARG;
    if (granularity < DMA_GRAN_TOKEN || granularity > DMA_GRAN_TENSOR) return DMA_ERR_INVALID_ARG;
    if (granularity == DMA_GRAN_BLOCK && block_rows <= 0) return DMA_ERR_INVALID_ARG;
    if (D != 64 && D != 128) return DMA_ERR_UNSUPPORTED;
    if (n_mat == 0 || S == 0) return DMA_OK;
    if (!x_bf16 || !amax_f32 || !aligned16(x_bf16) || (reinterpret_cast<uintptr_t>(amax_f32) & 3u) != 0) return DMA_ERR_INVALID_ARG;
    if (n_mat > ((int64_t)1 << 40) / S / D) return DMA_ERR_UNSUPPORTED;
    return dma::launch_group_amax(x_bf16, n_mat, S, D, is_query != 0, granularity, block_rows, (float*)amax_f32, (hipStream_t)stream);
}

int dma_mx_quantize_dual(const void* x_bf16, int64_t rows, int D, int is_query, void* codes_lo_u8,
                         void* scales_lo_u8, void* codes_hi_u8, void* scales_hi_u8, void* stream)
{
    int rc = check_quant_common(x_bf16, rows, D);
    if (rc != DMA_OK) return rc;
    if (rows == 0) return DMA_OK;
    if (!codes_lo_u8 || !scales_lo_u8 || !codes_hi_u8 || !scales_hi_u8) return DMA_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(codes_lo_u8) & 3u) != 0 || (reinterpret_cast<uintptr_t>(codes_hi_u8) & 7u) != 0)
        return DMA_ERR_INVALID_ARG;
    return dma::launch_mx_quantize(x_bf16, rows, D, 3, is_query != 0, codes_lo_u8, scales_lo_u8, codes_hi_u8,
                                   scales_hi_u8, nullptr, (hipStream_t)stream);
}

int dma_attn_fwd_ex(const void* q, const void* k, const void* v, void* out, int B, int Hq, int Hkv, int S,
                    int D, int causal, int diag_band_tiles, int hi_fmt, int lo_fmt, const dma_attn_opts* opts,
                    void* stream)
{
    if (!q || !k || !v || !out) return DMA_ERR_INVALID_ARG;
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || S <= 0 || D <= 0) return DMA_ERR_INVALID_ARG;
    if (Hq % Hkv != 0) return DMA_ERR_INVALID_ARG;
    if (diag_band_tiles < 0) return DMA_ERR_INVALID_ARG;
    if (!valid_fmt(hi_fmt) || !valid_fmt(lo_fmt)) return DMA_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out)) return DMA_ERR_INVALID_ARG;
    int tile = 128;
    int fp8_mfma = 0;
    int sink = 0;
    int per_token = 0;
    int pv_mx = 0;
    const float* q_amax = nullptr;
    const float* k_amax = nullptr;
    if (opts) {
        if (opts->fp8_mfma != 0 && opts->fp8_mfma != 1) return DMA_ERR_INVALID_ARG;
        fp8_mfma = opts->fp8_mfma;
        if (opts->tile != 0) tile = opts->tile;
        if (opts->tile < 0) return DMA_ERR_INVALID_ARG;
        if (opts->sink_tiles < 0) return DMA_ERR_INVALID_ARG;
        sink = opts->sink_tiles;
        if (opts->per_token_scale != 0 && opts->per_token_scale != 1) return DMA_ERR_INVALID_ARG;
        per_token = opts->per_token_scale;
        if ((opts->q_group_amax == nullptr) != (opts->k_group_amax == nullptr)) return DMA_ERR_INVALID_ARG;
        if (opts->q_group_amax && !per_token) return DMA_ERR_INVALID_ARG;
        if ((reinterpret_cast<uintptr_t>(opts->q_group_amax) & 3u) != 0 || (reinterpret_cast<uintptr_t>(opts->k_group_amax) & 3u) != 0) return DMA_ERR_INVALID_ARG;
        q_amax = (const float*)opts->q_group_amax;
        k_amax = (const float*)opts->k_group_amax;
        if (opts->pv_fmt != DMA_FMT_BF16 && opts->pv_fmt != DMA_FMT_MXFP8_E4M3) return DMA_ERR_UNSUPPORTED;
        pv_mx = opts->pv_fmt == DMA_FMT_MXFP8_E4M3;
    }
    if (tile != 64 && tile != 128) return DMA_ERR_UNSUPPORTED;
    // one head of the output must fit a 4 GiB buffer resource, rows of a partial or filled-up last tile group included
    // (their offsets must not wrap around before the resource's bounds drop them)
    if (((int64_t)S + 2 * tile) * D * 4 >= ((int64_t)1 << 32)) return DMA_ERR_UNSUPPORTED;
    if ((int64_t)B * Hq * S * D > (int64_t)1 << 40) return DMA_ERR_UNSUPPORTED;
    dma::AttnArgs a;
    a.q = q; a.k = k; a.v = v; a.out = (float*)out;
    a.B = B; a.Hq = Hq; a.Hkv = Hkv; a.S = S; a.D = D;
    a.tile = tile;
    const int n_tiles = (S + tile - 1) / tile;          // the last tile may be partial
    a.band = diag_band_tiles > n_tiles ? n_tiles : diag_band_tiles;
    a.sink = sink > n_tiles ? n_tiles : sink;
    a.causal = causal != 0;
    a.per_token = per_token;
    a.q_amax = q_amax;
    a.k_amax = k_amax;
    a.pv_mx = pv_mx;
    // the MX-format P V exists for the default pair (MXFP4 / MXFP8-E4M3 decoded exactly), without the per-token scale
    if (pv_mx && (per_token || fp8_mfma || lo_fmt != DMA_FMT_MXFP4_E2M1 || hi_fmt != DMA_FMT_MXFP8_E4M3)) return DMA_ERR_UNSUPPORTED;
    // public element format -> product path of the kernels: 3 / 4 = MXFP8 (E4M3 / E5M2) decoded exactly to bf16 and
    // multiplied on the bf16 MFMA; E5M2 has no other path
    if (fp8_mfma && (hi_fmt == DMA_FMT_MXFP8_E5M2 || lo_fmt == DMA_FMT_MXFP8_E5M2)) return DMA_ERR_UNSUPPORTED;
    if (fp8_mfma && per_token) return DMA_ERR_UNSUPPORTED;
    auto path = [&](int f) { return f == DMA_FMT_MXFP8_E5M2 ? 4 : (f == DMA_FMT_MXFP8_E4M3 && !fp8_mfma) ? 3 : f; };
    a.hi_fmt = path(hi_fmt);
    a.lo_fmt = path(lo_fmt);
    return dma::launch_attn_fwd(a, (hipStream_t)stream);
}

int dma_attn_fwd(const void* q, const void* k, const void* v, void* out, int B, int Hq, int Hkv, int S, int D,
                 int causal, int diag_band_tiles, int hi_fmt, int lo_fmt, void* stream)
{
    return dma_attn_fwd_ex(q, k, v, out, B, Hq, Hkv, S, D, causal, diag_band_tiles, hi_fmt, lo_fmt, nullptr, stream);
}

size_t dma_attn_fwd_workspace_bytes(int, int, int, int, int) { return 0; }

int dma_diag_copy(const void* src, void* dst, int64_t bytes, void* stream)
{
    if (bytes < 0 || bytes % 16 != 0) return DMA_ERR_INVALID_ARG;
    if (bytes == 0) return DMA_OK;
    if (!src || !dst || !aligned16(src) || !aligned16(dst)) return DMA_ERR_INVALID_ARG;
    return dma::launch_diag_copy(src, dst, bytes, (hipStream_t)stream);
}

int dma_diag_mfma(const void* a, const void* b, const void* a_scales, const void* b_scales, int fmt, void* out_f32, void* stream)
{
    if (fmt != DMA_FMT_BF16 && fmt != DMA_FMT_MXFP8_E4M3 && fmt != DMA_FMT_MXFP4_E2M1) return DMA_ERR_INVALID_ARG;
    if (!a || !b || !out_f32 || !aligned16(a) || !aligned16(b) || !aligned16(out_f32)) return DMA_ERR_INVALID_ARG;
    if (fmt != DMA_FMT_BF16 && (!a_scales || !b_scales)) return DMA_ERR_INVALID_ARG;
    return dma::launch_diag_mfma(a, b, a_scales, b_scales, fmt, (float*)out_f32, (hipStream_t)stream);     // public ids 0, 1, 2 = product paths 0, 1, 2
}

int dma_diag_pipes(const int* kinds, int n_slots, int microseconds, void* counts_u64, int* workgroups, void* stream)
{
    if (!kinds || !counts_u64 || n_slots < 1 || n_slots > 3 || microseconds < 1 || microseconds > 100000) return DMA_ERR_INVALID_ARG;
    if ((uintptr_t)counts_u64 % 8 != 0) return DMA_ERR_INVALID_ARG;
    for (int s = 0; s < n_slots; ++s)
        if (kinds[s] < DMA_PIPE_IDLE || kinds[s] > DMA_PIPE_CVT_PK_BF16) return DMA_ERR_INVALID_ARG;
    if (workgroups) {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return DMA_ERR_HIP;
        *workgroups = cus;
    }
    return dma::launch_diag_pipes(kinds, n_slots, 100LL * microseconds, (unsigned long long*)counts_u64, (hipStream_t)stream);
}

const char* dma_error_string(int code)
{
    switch (code) {
        case DMA_OK: return "ok";
        case DMA_ERR_INVALID_ARG: return "invalid argument (null or misaligned pointer, bad size or enum)";
        case DMA_ERR_UNSUPPORTED: return "valid request, but no kernel in this build covers it";
        case DMA_ERR_HIP: return "the HIP runtime reported an error at kernel launch";
    }
    return "unknown error code";
}

int dma_version(void) { return 100; }

}  // extern "C"
