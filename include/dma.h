/*
 * dma.h -- C ABI of the MI355X (gfx950) library for the fused forward pass of Diagonal-Tiled
 * Mixed-Precision Attention (DMA).
 *
 * Conventions for every call
 *   - Every data pointer is a DEVICE pointer owned by the caller (e.g. the storage of a PyTorch
 *     tensor); the library allocates nothing and writes only to the output buffers named below.  The only
 *     state it keeps between calls is read-only once filled: the compute-unit count per device and the
 *     number of resident workgroups per kernel instance, both queried from the runtime on first use.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls enqueue their
 *     kernels on it and return without waiting.  They issue nothing but kernel launches (no
 *     allocation, copy, memset or synchronisation), so a stream under HIP graph capture records
 *     them and the graph can be replayed.
 *   - Return value: DMA_OK (0) or a negative error code.  On error nothing has been enqueued.
 *     No C++ exception crosses the boundary.  dma_error_string() maps a code to a static string.
 *   - bf16 tensors are dense and row-major with the head dimension D innermost.
 *   - Inputs are assumed finite; NaN/Inf give unspecified results (never a fault).
 */
#ifndef DMA_H_
#define DMA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    DMA_OK = 0,
    DMA_ERR_INVALID_ARG = -1,   /* null pointer, non-positive size, bad enum value, misaligned pointer */
    DMA_ERR_UNSUPPORTED = -2,   /* a valid request this build has no kernel for */
    DMA_ERR_HIP = -3            /* the HIP runtime reported an error at launch */
};

/* Element formats.  MX formats carry one E8M0 scale byte per block of 32 consecutive elements
 * along D (paper, Table 1 and Sec. 3.1). */
enum {
    DMA_FMT_BF16 = 0,           /* no quantization: plain bf16 operands */
    DMA_FMT_MXFP8_E4M3 = 1,     /* FP8 E4M3 elements + E8M0 scale per 32 */
    DMA_FMT_MXFP4_E2M1 = 2,     /* FP4 E2M1 elements (two per byte) + E8M0 scale per 32 */
    DMA_FMT_MXFP8_E5M2 = 3      /* FP8 E5M2 elements + E8M0 scale per 32 (Sec. 4.2: e_max = 15) */
};

/*
 * MX quantization of a matrix (paper, Alg. 2 "Fused Mixed-Precision Quantization", Steps 1 and 3-7,
 * with the per-token scale of Step 2 equal to one; element encoding per Alg. 3 completed to a full
 * round-to-nearest-even).
 *
 *   x_bf16   [rows, D] bf16, device, read only.  16-byte aligned.
 *   rows     >= 0 (0 is a no-op).   D: multiple of 32, 32 <= D <= 1024.
 *   fmt      DMA_FMT_MXFP8_E4M3, DMA_FMT_MXFP8_E5M2 or DMA_FMT_MXFP4_E2M1.
 *   is_query non-zero: every element is first multiplied by log2(e)/sqrt(D) in one binary32
 *            multiplication (Alg. 2 Step 1).
 *   codes_u8 out, device.  E4M3, E5M2: [rows, D] bytes.  E2M1: [rows, D/2] bytes, element 2t in the low
 *            nibble and 2t+1 in the high nibble (Alg. 2 Step 5).
 *   scales_u8 out, device, [rows, D/32] bytes: clamp(floor(log2 max|block|) - e_max + 127, 0, 254)
 *            with e_max = 8 (E4M3), 15 (E5M2) or 2 (E2M1) (Alg. 2 Steps 6-7); an all-zero block gives 0.
 *   Element = round-to-nearest-even of x / 2^(scale-127) after clamping to +-448 / +-57344 / +-6; the sign bit
 *   is the sign bit of x even when the magnitude rounds to zero.
 */
int dma_mx_quantize(const void* x_bf16, int64_t rows, int D, int fmt, int is_query,
                    void* codes_u8, void* scales_u8, void* stream);

/* dma_mx_quantize with Step 2 of Alg. 2 applied (the "Per-Token" granularity of Sec. 5.3): every row is first divided
 * by S_q = max_D|x| / (448 * 6) (as one binary32 multiplication by 2688 / max), then quantized as above;
 * token_scales_f32 [rows] float32, device, out, receives S_q (the dequantized row is decode * 2^(scale-127) * S_q).
 * Rows whose maximum is below 2^-100 keep S_q = 1.  D / 8 must be a power of two <= 64 (D in 32, 64, 128, 256, 512),
 * else DMA_ERR_UNSUPPORTED. */
int dma_mx_quantize_token(const void* x_bf16, int64_t rows, int D, int fmt, int is_query,
                          void* codes_u8, void* scales_u8, void* token_scales_f32, void* stream);

/* The same with both formats produced from ONE read of x (the "MP" fusion of Alg. 2: low copy =
 * MXFP4 E2M1, high copy = MXFP8 E4M3).  Buffers as above. */
int dma_mx_quantize_dual(const void* x_bf16, int64_t rows, int D, int is_query,
                         void* codes_lo_u8, void* scales_lo_u8,
                         void* codes_hi_u8, void* scales_hi_u8, void* stream);

/*
 * Fused DMA forward (paper, Alg. 1 "Diagonal-Tiled Mixed-Precision Attention" with the online
 * softmax of Sec. 3.2, and the quantization of Alg. 2 done inside the kernel).
 *
 *   q   [B, Hq,  S, D] bf16      k, v [B, Hkv, S, D] bf16      out [B, Hq, S, D] float32
 *   All device, dense, 16-byte aligned.  Hq % Hkv == 0; query head h reads kv head h / (Hq/Hkv).
 *   causal            non-zero: Alg. 1 (key tiles jt <= it, keys after the query masked on the diagonal tile).
 *                     zero: every key tile is visited and nothing is masked (Sec. 4.1, "Compatibility with
 *                     Non-Causal Attention").
 *   diag_band_tiles   b = T / B_N >= 0.  For the query tile `it`, key tile `jt` is computed in hi_fmt iff
 *                     it - jt < b (causal) or |it - jt| < b (non-causal), otherwise in lo_fmt.  b = 0: every
 *                     tile in lo_fmt; b >= S/tile: every tile in hi_fmt.
 *   hi_fmt, lo_fmt    DMA_FMT_* for the Q K^T product of the tiles in / outside the diagonal band.
 *                     Supported pairs (lo, hi): (E2M1, E4M3), (E2M1, E5M2), (E2M1, E2M1), (E4M3, E4M3),
 *                     (E5M2, E5M2), (BF16, BF16); any other pair returns DMA_ERR_UNSUPPORTED.
 *   Key tiles are visited in ascending order in every variant.
 *   The logical tile is B_M = B_N = 128 for dma_attn_fwd and D must be 128.  S >= 1 is arbitrary: the last tile may be
 *   partial (Sec. 3.2 tiles the sequence with a ceiling); keys past the end do not exist and rows past the end are
 *   not written.  (S + 2 * tile) * D * 4 must stay below 4 GiB (else DMA_ERR_UNSUPPORTED).
 *
 *   Per key tile: scores in base 2 (the factor log2(e)/sqrt(D) is folded into Q before quantization;
 *   for BF16 it multiplies the binary32 score), keys after the query masked to -inf on the diagonal
 *   tile, running maximum / sum in binary32, probabilities rounded to bf16 for the P V product
 *   (V stays bf16), binary32 accumulation, final division by the running sum.  No intermediate is
 *   written to device memory.
 */
int dma_attn_fwd(const void* q, const void* k, const void* v, void* out,
                 int B, int Hq, int Hkv, int S, int D, int causal,
                 int diag_band_tiles, int hi_fmt, int lo_fmt, void* stream);

/* Options for dma_attn_fwd_ex.  Zero-initialise, then set fields. */
typedef struct dma_attn_opts {
    int tile;             /* logical tile B_M = B_N: 128 (with D = 128) or 64 (with D = 64); 0 = 128 */
    int sink_tiles;       /* >= 0: the first sink_tiles key tiles are computed in hi_fmt for every query tile (Sec. 5.3,
                             the sink window of the diagonal/sink table); 0 = Alg. 1 as printed */
    int pv_fmt;           /* DMA_FMT_BF16 (default): V and P stay 16-bit, as in Alg. 1.
                             DMA_FMT_MXFP8_E4M3: an extension beyond the paper: P (per key tile, masked keys as 0) and V are
                             quantized to MXFP8-E4M3 with one E8M0 scale per 32 consecutive keys (rule of Alg. 2 Steps 6-7) and
                             multiplied on the block-scaled FP8 MFMA; the row sum still adds the unrounded probabilities.
                             Only with lo_fmt = MXFP4_E2M1, hi_fmt = MXFP8_E4M3, fp8_mfma = 0, per_token_scale = 0; slower
                             than the default on gfx950.  Any other value: DMA_ERR_UNSUPPORTED */
    int per_token_scale;  /* 0: Alg. 2 Step 2 is the identity (default).  1: queries and keys go through Step 2 (row divided by
                             S_q = rowmax / 2688 before quantization) and the score product is multiplied by S_q of its
                             query and of its key; ignored for DMA_FMT_BF16 operands; not with fp8_mfma = 1 */
    const void* q_group_amax;  /* only with per_token_scale = 1; device float32, 4-byte aligned.  NULL (default): per-token
                             granularity, the scale of a row comes from its own maximum.  Otherwise q_group_amax [B, Hq, S]
                             and k_group_amax [B, Hkv, S] (both or neither) give, for every query / key row, the maximum
                             magnitude of the group of rows that shares its Step-2 scale (Sec. 5.3 names per-block and
                             per-tensor granularities): S_q = that maximum / 2688.  dma_mx_group_amax produces them */
    const void* k_group_amax;
    int fp8_mfma;         /* how MXFP8 tiles form Q K^T.
                             0 (default): the E4M3 codes and E8M0 scales are decoded exactly to bf16 and
                               multiplied on the bf16 MFMA: the product of the quantized operands is exact up to
                               binary32 accumulation, as the method defines it.
                             1: the codes and scales go to the block-scaled FP8 MFMA.  That instruction adds the
                               products of 8 consecutive elements along D in a short fixed-point adder: each is aligned
                               to the largest of its group and cut off below 2^-13 of that product's leading bit (the
                               groups' sums are then added in binary32), so a score dominated by a few large products
                               -- an outlier channel -- is off by up to 7 * 2^-13 of them per group
                               (tests/test_gpu_mfma_accumulation.py establishes this through dma_diag_mfma); twice the
                               matrix rate of mode 0 on those tiles, looser parity.
                             MXFP4 tiles always use the block-scaled FP4 MFMA, which sums exactly. */
} dma_attn_opts;

/*
 * Group maxima for Alg. 2 Step 2 at a granularity coarser than the row (Sec. 5.3, table of quantization granularities:
 * per-tensor, per-block, per-token; the paper names them without defining the groups).
 *   x_bf16    [n_mat, S, D] bf16, device, 16-byte aligned; D = 64 or 128 (the head dimensions dma_attn_fwd_ex takes).
 *   amax_f32  [n_mat * S] float32, device: for every row the largest magnitude (if is_query: after the binary32
 *             multiplication by log2(e)/sqrt(D) of Alg. 2 Step 1) within the row's group.
 *   granularity  DMA_GRAN_TOKEN: the row itself; DMA_GRAN_BLOCK: block_rows (> 0) consecutive rows of one [S, D] matrix,
 *             blocks starting at multiples of block_rows (the last one may be shorter); DMA_GRAN_TENSOR: all of x.
 * Two to four small kernels on `stream`; no allocation.
 */
#define DMA_GRAN_TOKEN 1
#define DMA_GRAN_BLOCK 2
#define DMA_GRAN_TENSOR 3
int dma_mx_group_amax(const void* x_bf16, int64_t n_mat, int64_t S, int D, int is_query, int granularity,
                      int64_t block_rows, void* amax_f32, void* stream);

/* dma_attn_fwd with explicit options; opts == NULL means the defaults of dma_attn_fwd. */
int dma_attn_fwd_ex(const void* q, const void* k, const void* v, void* out,
                    int B, int Hq, int Hkv, int S, int D, int causal,
                    int diag_band_tiles, int hi_fmt, int lo_fmt,
                    const dma_attn_opts* opts, void* stream);

/* Device scratch the forward needs beyond its inputs and output: always 0. */
size_t dma_attn_fwd_workspace_bytes(int B, int Hq, int Hkv, int S, int D);

/* Diagnostic, not part of the method: plain device-to-device copy kernel (16 bytes per lane, no reuse) of `bytes`
 * bytes (a multiple of 16; src, dst 16-byte aligned, device, non-overlapping).  Its exactly known traffic (bytes read +
 * bytes written) is what the HBM byte counters of a profiler run are scaled by. */
int dma_diag_copy(const void* src, void* dst, int64_t bytes, void* stream);

/* Diagnostic, not part of the method: ONE 32 x 32 x 64 product out[i][j] = sum_k a[i][k] * b[j][k] on the matrix
 * instruction of the named format, operands exactly as given -- the evidence behind opts.fp8_mfma (what the block-scaled
 * FP8 instruction does with the small products of a block next to a large one; tests/test_gpu_mfma_accumulation.py).
 *   fmt       DMA_FMT_MXFP8_E4M3 / DMA_FMT_MXFP4_E2M1: the block-scaled instruction; DMA_FMT_BF16: four k = 16 steps
 *             of the bf16 instruction.
 *   a, b      device, 16-byte aligned, row-major [32][64] elements along k: E4M3 one byte each; E2M1 two per byte
 *             (even k in the low nibble), i.e. [32][32] bytes; bf16 two bytes each.
 *   a_scales, b_scales   device, [32][2] E8M0 bytes (row, 32-element block); ignored (may be NULL) for DMA_FMT_BF16.
 *   out_f32   device, 16-byte aligned, [32][32] float32. */
int dma_diag_mfma(const void* a, const void* b, const void* a_scales, const void* b_scales, int fmt,
                  void* out_f32, void* stream);

/* Diagnostic, not part of the method: the rates pure instruction streams reach side by side on one SIMD -- the evidence
 * for how much of the matrix time of the forward can hide behind its vector work.  One workgroup per compute unit;
 * wave slot s (waves 4 s .. 4 s + 3 of the workgroup, one on each SIMD) issues the stream kinds[s] back to back for
 * `microseconds` and adds the number of instructions it issued to counts_u64[s]; the waves stop by the clock.
 *   kinds       host, n_slots ints (1 <= n_slots <= 3), each a DMA_PIPE_* id
 *   microseconds  1 .. 100 000
 *   counts_u64  device, 8-byte aligned, 3 x uint64, zeroed by the caller before the call; slot s receives the sum over
 *               all its waves (4 per workgroup)
 *   workgroups  host, may be NULL: receives the number of workgroups launched (the compute units of the device)
 * Clocks per instruction of slot s = microseconds x clock [MHz] x 4 x workgroups / counts_u64[s]. */
#define DMA_PIPE_IDLE 0
#define DMA_PIPE_MFMA_BF16 1        /* v_mfma_f32_32x32x16_bf16 */
#define DMA_PIPE_MFMA_FP4 2         /* v_mfma_scale_f32_32x32x64_f8f6f4, E2M1 operands */
#define DMA_PIPE_MFMA_FP8 3         /* the same instruction, E4M3 operands */
#define DMA_PIPE_FMA 4              /* v_fma_f32 */
#define DMA_PIPE_EXP 5              /* v_exp_f32 */
#define DMA_PIPE_CVT_PK_BF16 6      /* v_cvt_pk_bf16_f32 */
int dma_diag_pipes(const int* kinds, int n_slots, int microseconds, void* counts_u64, int* workgroups, void* stream);

/* Static, NUL-terminated description of a return code. */
const char* dma_error_string(int code);

/* Library version: major * 10000 + minor * 100 + patch. */
int dma_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DMA_H_ */
