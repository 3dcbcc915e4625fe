// Fused forward: dispatch over the (low format, high format) pairs.  The kernel lives in dma_attn_kernel.hpp; each
// pair is its own object file (dma_attn_inst.hip).
#include "dma_device.hpp"
#include "dma_internal.hpp"

namespace dma {

// (lo, hi) product-path ids; the list the build compiles dma_attn_inst.hip for.
int launch_attn_pair_2_3(const AttnArgs&, hipStream_t);    // MXFP4 / MXFP8-E4M3 decoded to bf16   (the DMA default)
int launch_attn_pair_2_1(const AttnArgs&, hipStream_t);    // MXFP4 / MXFP8-E4M3 on the FP8 MFMA
int launch_attn_pair_2_4(const AttnArgs&, hipStream_t);    // MXFP4 / MXFP8-E5M2 decoded to bf16
int launch_attn_pair_2_2(const AttnArgs&, hipStream_t);    // all MXFP4
int launch_attn_pair_3_3(const AttnArgs&, hipStream_t);    // all MXFP8-E4M3 decoded to bf16
int launch_attn_pair_1_1(const AttnArgs&, hipStream_t);    // all MXFP8-E4M3 on the FP8 MFMA
int launch_attn_pair_4_4(const AttnArgs&, hipStream_t);    // all MXFP8-E5M2 decoded to bf16
int launch_attn_pair_0_0(const AttnArgs&, hipStream_t);    // unquantized bf16 baseline

int launch_attn_fwd(const AttnArgs& a, hipStream_t stream)
{
    const int lo = a.lo_fmt, hi = a.hi_fmt;       // product-path ids (FMT_*)
    if (lo == FMT_E2M1 && hi == FMT_E4M3_X) return launch_attn_pair_2_3(a, stream);
    if (lo == FMT_E2M1 && hi == FMT_E4M3) return launch_attn_pair_2_1(a, stream);
    if (lo == FMT_E2M1 && hi == FMT_E5M2_X) return launch_attn_pair_2_4(a, stream);
    if (lo == FMT_E2M1 && hi == FMT_E2M1) return launch_attn_pair_2_2(a, stream);
    if (lo == FMT_E4M3_X && hi == FMT_E4M3_X) return launch_attn_pair_3_3(a, stream);
    if (lo == FMT_E4M3 && hi == FMT_E4M3) return launch_attn_pair_1_1(a, stream);
    if (lo == FMT_E5M2_X && hi == FMT_E5M2_X) return launch_attn_pair_4_4(a, stream);
    if (lo == FMT_BF16 && hi == FMT_BF16) return launch_attn_pair_0_0(a, stream);
    return DMA_ERR_UNSUPPORTED_;
}

}  // namespace dma
