// One (low format, high format) pair of the fused forward: compiled once per pair with -DDMA_LO=<id> -DDMA_HI=<id>
// (product-path ids of dma_device.hpp), so that the pairs build in parallel.  Defines
// dma::launch_attn_pair_<LO>_<HI>(), which picks the tile shape.
#include "dma_attn_kernel.hpp"

#if !defined(DMA_LO) || !defined(DMA_HI)
#error "compile with -DDMA_LO=<format id> -DDMA_HI=<format id>"
#endif

#define DMA_PASTE3(a, b, c, d) a##b##c##d
#define DMA_PAIR_NAME(lo, hi) DMA_PASTE3(launch_attn_pair_, lo, _, hi)

namespace dma {

int DMA_PAIR_NAME(DMA_LO, DMA_HI)(const AttnArgs& a, hipStream_t stream)
{
    if (a.D == 128 && a.tile == 128) {
        // two logical tiles per workgroup (256 query rows share each K/V tile); with an odd number of tiles the last
        // pair is filled up with a tile past the end of the sequence.  One tile per workgroup only for a single tile.
        if (a.S > 128) return launch_instance<128, 128, 2, DMA_LO, DMA_HI>(a, stream);
        return launch_instance<128, 128, 1, DMA_LO, DMA_HI>(a, stream);
    }
    if (a.D == 64 && a.tile == 64) {
        if (a.S > 64) return launch_instance<64, 64, 2, DMA_LO, DMA_HI>(a, stream);
        return launch_instance<64, 64, 1, DMA_LO, DMA_HI>(a, stream);
    }
    return DMA_ERR_UNSUPPORTED_;
}

}  // namespace dma
