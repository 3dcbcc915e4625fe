// Fused forward of Diagonal-Tiled Mixed-Precision Attention for gfx950 (paper, Alg. 1 with the
// online softmax of Sec. 3.2; Q/K quantization of Alg. 2 done in-kernel; options: sink window and
// per-token scale of Sec. 5.3, non-causal variant of Sec. 4.1).
//
// Work split.  A work item is TPW consecutive logical query tiles (B_M = BT rows each) of one
// (batch, query head); the workgroup that owns it walks the key tiles jt = 0, 1, ... in ascending
// order, so one K/V tile fetched and quantized once serves TPW * BT query rows.  Each wave owns 32
// query rows of one logical tile `it` and follows Alg. 1 for that tile: key tiles before the
// diagonal band in the low format (Phase 1), the last `band` tiles up to the diagonal one in the
// high format (Phase 2), tiles after its diagonal are skipped.  The grid is one resident workgroup
// per CU; each walks a static, balanced list of items (see the kernel).
//
// Everything is computed transposed so that a query row lives in one lane column:
//     S^T[key, query] = K . Q^T      block-scaled MFMA 32x32x64 (A = K codes from LDS, B = Q codes in VGPRs)
//                                     or bf16 MFMA 32x32x16 for the exact MXFP8 / unquantized paths
//     O^T[d,  query] += V^T . P^T    bf16 MFMA 32x32x16 (A = V^T via LDS transpose reads, B = P^T = the
//                                     exponentiated S^T accumulators, already in operand layout)
// so the row maximum / sum need one cross-half exchange and the running state (m, l) is per lane.
//
// Pipeline.  K and V of tile jt+2 are in flight from global memory (16 B per lane, coalesced) while
// tile jt is computed out of LDS buffer jt & 1 and tile jt+1 is quantized (block maximum over a lane
// quad by DPP, E8M0 scale, hardware scaled converts) into buffer (jt+1) & 1: one barrier per tile.
// Two waves per SIMD (the register budget allows no more): the matrix work of one overlaps the vector
// work of the other, and together they reach the full vector issue rate, which one wave alone does not.
#pragma once

#include <atomic>
#include "dma_device.hpp"
#include "dma_internal.hpp"

namespace dma {

template <int A, int B>
constexpr int cmax() { return A > B ? A : B; }

template <int D_, int BT_, int TPW_>
struct Cfg {
    static constexpr int D = D_, BT = BT_, TPW = TPW_;
    static constexpr int WPT = BT / 32;          // waves per logical query tile (32 rows each)
    static constexpr int NW = WPT * TPW;         // waves per workgroup
    static constexpr int T = NW * 64;            // threads per workgroup
    static constexpr int NKB = BT / 32;          // 32-key blocks per key tile
    static constexpr int NDB = D / 32;           // 32-wide blocks of the head dimension (output)
    static constexpr int NH = D / 64;            // k=64 scaled MFMAs per score block
    static constexpr int NKK = D / 16;           // k=16 bf16 MFMAs per score block
    static constexpr int CPR = D / 8;            // 16-byte chunks per row
    static constexpr int CH = BT * CPR;          // chunks per tile
    static constexpr int CPT = CH / T;           // chunks per thread
    static_assert(CH % T == 0, "tile must split evenly over the threads");
    static_assert(D % 64 == 0, "head dimension must be a multiple of 64");
    // LDS row strides in bytes; the padding spreads consecutive rows over the banks.
    static constexpr int KS4 = D / 2 + 16;       // E2M1 codes
    static constexpr int KS8 = D + 16;           // E4M3 codes
    static constexpr int KSB = 2 * D + 16;       // bf16 keys
    static constexpr int VS = 2 * D;             // bf16 values: dense rows, 16-byte chunks XOR-swizzled (see v_swizzle)
    static constexpr int KSC = BT * CPR;         // scale bytes of one tile: one per 16-byte chunk (each block's 4 chunks repeat its code)
    static constexpr int VBYTES = BT * VS;
    // MX-format P V: V as E4M3 codes, one byte per element in padded rows, then one scale byte per (32-key block,
    // column).  In its staging each wave owns the keys of one 32-key block (and, with two logical tiles per workgroup,
    // half of the columns), so that the block maxima along the key axis never leave the wave.
    static constexpr int VS8 = D + 16;
    static constexpr int V8CODES = BT * VS8;
    static constexpr int V8BYTES = V8CODES + NKB * D;
    static constexpr int VCW = CPR / TPW;        // 16-byte chunks (of 8 columns) per row of lanes
    static constexpr int VRG = 64 / VCW;         // keys per chunk round of a wave
    static_assert(NW == NKB * TPW && VRG * CPT == 32, "one 32-key block per wave (and column half)");
    // V rows sit densely in LDS; so that the transpose reads of four consecutive keys do not hit the same banks,
    // chunk c of key k is stored at chunk c ^ (4 * v_swizzle(k)).
    static constexpr int v_swizzle(int key) { return D == 128 ? (key & 3) : ((key >> 1) & 1); }
    template <int FMT>
    static constexpr int kstride() { return FMT == FMT_E2M1 ? KS4 : FMT == FMT_E4M3 ? KS8 : KSB; }
    template <int FMT>
    static constexpr int kbytes() { return BT * kstride<FMT>(); }
    // Query operand storage in 16-byte units: scaled MFMA: NH x (4 or 8 dwords); bf16 MFMA: NKK x 4 dwords.
    template <int FMT>
    static constexpr int qregs() { return FMT == FMT_E2M1 ? NH : FMT == FMT_E4M3 ? 2 * NH : NKK; }
};

// ---------------------------------------------------------------------------------------------
// Query operand of a wave: its 32 rows in MFMA B-operand layout.  Lane (j, g) = (lane % 32, lane / 32) owns row j and
// the MX blocks 2h + g (h < NH) of that row: raw[4h + t] is the 16-byte chunk t of block 2h + g, i.e. elements
// 32 (2h + g) + 8t + [0, 8).  Every format's operand is made from these registers, so one set of loads serves both
// precisions and every block maximum is lane-local:
//   scaled MFMA (k = 64 per step h): block 2h + g is exactly the lane's share of step h;
//   bf16 MFMA (k = 16 per step kk = 4h + t): the lane's 8 elements of step kk are chunk t of block 2h + g -- a
//   permutation of the head dimension against the instruction's natural order, which the K side mirrors (see score_part).
// ---------------------------------------------------------------------------------------------
// Global memory goes through buffer resources whose size is the valid part of the [S, D] matrix: a 16-byte access
// past row S - 1 is out of range for the hardware bounds check, reads as zero and is dropped on a store, so a partial
// last tile needs no address guards.  Only the per-lane offset operand takes part in that check (the scalar offset
// operand does not), so everything that can run past the end is in the per-lane offset or in the resource's base.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
DMA_DEV rsrc_t make_rsrc(const void* base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);   // raw dword buffer
}
DMA_DEV v4i buffer_load16(rsrc_t r, unsigned byte_offset)
{
    return __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(r, (int)byte_offset, 0, 0));
}
DMA_DEV void buffer_store16(rsrc_t r, unsigned byte_offset, v4f v)
{
    // non-temporal: the output is written once and read by nobody here, it should not push K/V lines out of the L2
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4u, v), r, (int)byte_offset, 0, 2);
}

// qmat: the [S, D] bf16 query matrix of the head (resource over its S rows); rows >= S read as zero.
template <typename C>
DMA_DEV void load_q_raw(v4i (&raw)[C::NKK], rsrc_t qmat, int row0, int j, int g)
{
    const unsigned off = (unsigned)(row0 + j) * (C::D * 2) + 64 * g;
#pragma unroll
    for (int h = 0; h < C::NH; ++h)
#pragma unroll
        for (int t = 0; t < 4; ++t) raw[4 * h + t] = buffer_load16(qmat, off + 128 * h + 16 * t);
}

// Absolute maximum of the lane's query row after the softmax pre-scale (both half-waves hold half of the row).
template <typename C>
DMA_DEV float q_row_amax(const v4i (&raw)[C::NKK], float c)
{
    float amax = 0.f;
#pragma unroll
    for (int kk = 0; kk < C::NKK; ++kk) {
        float x[8];
        unpack8<true>(raw[kk], c, x);
        amax = fmaxf(amax, amax8(x));
    }
    return cross_half_max(amax);
}

// qr / qscale from raw (scaled MFMA formats fill `qscale`: byte h = E8M0 of block 2h + g of the lane's row).
// inv_sq: the factor 1 / S_q of Alg. 2 Step 2 for the lane's row (1 when the per-token scale is off): one more
// binary32 multiply per element before the shared scales are formed.
template <typename C, int FMT, bool PT, int QR>
DMA_DEV void make_q(v4i (&qr)[QR], int& qscale, const v4i (&raw)[C::NKK], float c, float inv_sq)
{
    qscale = 0;
    if constexpr (FMT == FMT_BF16) {
#pragma unroll
        for (int kk = 0; kk < C::NKK; ++kk) qr[kk] = raw[kk];
    } else {
        static_for<C::NH>([&](auto H) {
            constexpr int h = H;
            float x[4][8];
            float amax = 0.f;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                unpack8<true>(raw[4 * h + t], c, x[t]);
                if constexpr (PT) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) x[t][e] = __fmul_rn(x[t][e], inv_sq);
                }
                amax = fmaxf(amax, amax8(x[t]));
            }
            const int code = e8m0_code<FMT>(amax);
            if constexpr (FMT == FMT_E4M3_X || FMT == FMT_E5M2_X) {
#pragma unroll
                for (int t = 0; t < 4; ++t) qr[4 * h + t] = quant_dequant8<FMT>(x[t], code);
            } else if constexpr (FMT == FMT_E2M1) {
                qscale |= code << (8 * h);
                v4i r;
#pragma unroll
                for (int t = 0; t < 4; ++t) r[t] = encode8_e2m1(x[t], code);
                qr[h] = r;
            } else {
                qscale |= code << (8 * h);
                int r[8];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const v2i e = encode8_e4m3(x[t], code);
                    r[2 * t] = e[0];
                    r[2 * t + 1] = e[1];
                }
                // E4M3 operand layout: VGPR 0-3 = first half of block 2h (lower lanes) / second half of
                // block 2h (upper lanes); VGPR 4-7 the same for block 2h+1.  Each lane encoded one whole
                // block, so the lower lanes' VGPR 4-7 trade places with the upper lanes' VGPR 0-3.
#pragma unroll
                for (int t = 0; t < 4; ++t) swap_halves(r[t], r[4 + t]);
                qr[2 * h] = v4i{r[0], r[1], r[2], r[3]};
                qr[2 * h + 1] = v4i{r[4], r[5], r[6], r[7]};
            }
        });
    }
}

// ---------------------------------------------------------------------------------------------
// LDS addressing.  All LDS traffic goes through 32-bit byte addresses of the form
// (one pinned per-lane VGPR) + (compile-time constant), so every access uses the instruction's immediate
// offset and the loops carry a handful of address registers instead of one per access.
// ---------------------------------------------------------------------------------------------
#define DMA_LDS __attribute__((address_space(3)))
DMA_DEV unsigned pin(unsigned x) { asm volatile("" : "+v"(x)); return x; }
// Lane / thread index made opaque at the point of use: the address arithmetic that follows is then redone where
// it is needed (a few integer ops) instead of being hoisted out of the tile loops into long-lived registers.
DMA_DEV int fresh(int x) { asm volatile("" : "+v"(x)); return x; }
template <typename T>
DMA_DEV T lds_read(unsigned addr) { return *(const DMA_LDS T*)(uintptr_t)addr; }
template <typename T>
DMA_DEV void lds_write(unsigned addr, T v) { *(DMA_LDS T*)(uintptr_t)addr = v; }
DMA_DEV v4s lds_read_tr16(unsigned addr) { return __builtin_amdgcn_ds_read_tr16_b64_v4i16((DMA_LDS v4s*)(uintptr_t)addr); }
DMA_DEV v2i lds_read_tr8(unsigned addr) { return __builtin_amdgcn_ds_read_tr8_b64_v2i32((DMA_LDS v2i*)(uintptr_t)addr); }

// ---------------------------------------------------------------------------------------------
// Staging of one key/value tile
// ---------------------------------------------------------------------------------------------
// The lane-dependent parts of the LDS addresses of a step never change during the kernel: the low-format ones are
// computed once (LaneOffsets) and every step only adds the uniform buffer base; the high-format ones, used on a few
// tiles per item, are recomputed where they are needed.
template <typename C, int FMT>
DMA_DEV unsigned stage_k_lane(int tid)           // where the thread's first chunk of a K tile goes (codes)
{
    constexpr int CB = (FMT == FMT_E2M1) ? 4 : (FMT == FMT_E4M3) ? 8 : 16;     // bytes per chunk in LDS
    return (tid / C::CPR) * C::template kstride<FMT>() + (tid % C::CPR) * CB;
}
template <typename C>
DMA_DEV unsigned stage_s_lane(int tid) { return (tid / C::CPR) * C::CPR + tid % C::CPR; }   // ... its scale byte
template <typename C>
DMA_DEV unsigned stage_v_lane(int tid)           // ... its first chunk of a V tile (swizzled, see Cfg::v_swizzle)
{
    const int key0 = tid / C::CPR, dc = tid % C::CPR;
    return key0 * C::VS + ((dc ^ (4 * C::v_swizzle(key0))) * 16);
}
template <typename C, int FMT>
DMA_DEV unsigned score_k_lane(int lane)          // the lane's key row of 32-key block 0 (K operand reads)
{
    // the bf16 MFMA paths read the head dimension in the query operand's order
    return (lane & 31) * C::template kstride<FMT>() + (uses_bf16_mfma(FMT) ? 64 : 16) * (lane >> 5);
}
template <typename C>
DMA_DEV unsigned score_s_lane(int lane) { return (lane & 31) * C::CPR + 4 * (lane >> 5); }  // ... its scale dword
// Transpose read of V: lane l16 of a 16-lane group points at row (l16 / 4) of a 4-key x 16-column patch; the row's
// 16-byte chunks are swizzled by the row index (the same for every patch: patches start at multiples of 4).
template <typename C>
DMA_DEV unsigned value_v_lane(int lane, int db)  // the lane's address for d-block db in the tile's first patch
{
    const int g = lane >> 5, l16 = lane & 15, q16 = lane >> 4;
    const unsigned row_off = (4 * g + (l16 >> 2)) * C::VS + 8 * (l16 & 1);
    return row_off + 16 * ((4 * db + 2 * (q16 & 1) + ((l16 & 3) >> 1)) ^ (4 * C::v_swizzle(l16 >> 2)));
}
// MX-format P V.  Thread -> (32-key block kb, key in the block, 16-byte chunk of the row) of its round-0 chunk; round r
// is VRG keys further on.
template <typename C>
DMA_DEV void vmx_thread(int tid, int& kb, int& key, int& chunk)
{
    const int w = tid >> 6, ln = tid & 63;
    kb = w % C::NKB;
    key = ln / C::VCW;
    chunk = C::VCW * (w / C::NKB) + ln % C::VCW;
}
// Transpose read of the E4M3 V tile: lanes 2 r and 2 r + 1 of a 16-lane group point at the halves of 16 columns of key
// row f(r) = r (r < 4) or r + 4 (r >= 4), plus 4 for the upper half-wave: read 0 then delivers, byte by byte, the keys
// 8 v + 4 g + b of VGPRs v = 0, 1 of the operand; the other reads are 16, 32 and 48 keys further on.
template <typename C>
DMA_DEV unsigned value_vmx_lane(int lane)
{
    const int g = lane >> 5, l16 = lane & 15, q16 = (lane >> 4) & 1, r = l16 >> 1;
    return (4 * g + (r < 4 ? r : r + 4)) * C::VS8 + 16 * q16 + 8 * (l16 & 1);
}
template <typename C, int LO>
struct LaneOffsets {
    unsigned stage_k, stage_s, stage_v, score_k, score_s, value_v[C::NDB];
    DMA_DEV void init(int tid, int lane)
    {
        stage_k = pin(stage_k_lane<C, LO>(tid));
        stage_s = pin(stage_s_lane<C>(tid));
        stage_v = pin(stage_v_lane<C>(tid));
        score_k = pin(score_k_lane<C, LO>(lane));
        score_s = pin(score_s_lane<C>(lane));
#pragma unroll
        for (int db = 0; db < C::NDB; ++db) value_v[db] = pin(value_v_lane<C>(lane, db));
    }
};

// Chunk r of thread tid is 16-byte chunk r * T + tid of the dense tile: key r * (T / CPR) + tid / CPR.
template <typename C, bool BOUNDED>
DMA_DEV void load_tile(v4i (&reg)[C::CPT], const uint16_t* __restrict__ mat, int row0, int S, int tid)
{
    // rows [row0, row0 + BT) of the [S, D] bf16 matrix `mat` (uniform).  BOUNDED: rows >= S read as zero; otherwise
    // the caller guarantees row0 + BT <= S.
    constexpr int KPR = C::T / C::CPR;                       // rows per chunk round
    const unsigned lane_off = (unsigned)fresh(tid) * 16u;
    if constexpr (!BOUNDED) {
        // whole tile: plain loads in the (scalar base + 32-bit lane offset) form; the bases are pinned in scalar
        // registers so that no vector address arithmetic is generated
        typedef const __attribute__((address_space(1))) v4i* global_v4i;
#pragma unroll
        for (int r = 0; r < C::CPT; ++r) {
            const uint64_t t64 = (uint64_t)(mat + (int64_t)row0 * C::D) + (uint64_t)r * C::T * 16;
            uint32_t lo = (uint32_t)t64, hi = (uint32_t)(t64 >> 32);
            asm volatile("" : "+s"(lo), "+s"(hi));
            reg[r] = *(global_v4i)((((uint64_t)hi << 32) | (uint64_t)lo) + (uint64_t)lane_off);
        }
    } else {
        // one buffer resource per chunk round, based at the round's first row and as long as what is left of the
        // matrix from there
#pragma unroll
        for (int r = 0; r < C::CPT; ++r) {
            const int row = row0 + r * KPR;
            const int64_t left = (int64_t)(S - row) * (C::D * 2);
            const rsrc_t rs = make_rsrc(mat + (int64_t)row * C::D, left > 0 ? (uint32_t)left : 0u);
            reg[r] = buffer_load16(rs, lane_off);
        }
    }
}

// V tile in the thread mapping of the MX-format P V (vmx_thread).
template <typename C, bool BOUNDED>
DMA_DEV void load_tile_vmx(v4i (&reg)[C::CPT], const uint16_t* __restrict__ mat, int row0, int S, int tid)
{
    int kb, key, chunk;
    vmx_thread<C>(fresh(tid), kb, key, chunk);
    const unsigned lane_off = (unsigned)((32 * kb + key) * C::CPR + chunk) * 16u;     // < BT * D * 2: inside the tile
    if constexpr (!BOUNDED) {
        typedef const __attribute__((address_space(1))) v4i* global_v4i;
#pragma unroll
        for (int r = 0; r < C::CPT; ++r) {
            const uint64_t t64 = (uint64_t)(mat + (int64_t)(row0 + r * C::VRG) * C::D);
            uint32_t lo = (uint32_t)t64, hi = (uint32_t)(t64 >> 32);
            asm volatile("" : "+s"(lo), "+s"(hi));
            reg[r] = *(global_v4i)((((uint64_t)hi << 32) | (uint64_t)lo) + (uint64_t)lane_off);
        }
    } else {
#pragma unroll
        for (int r = 0; r < C::CPT; ++r) {
            const int row = row0 + r * C::VRG;
            const int64_t left = (int64_t)(S - row) * (C::D * 2);
            const rsrc_t rs = make_rsrc(mat + (int64_t)row * C::D, left > 0 ? (uint32_t)left : 0u);
            reg[r] = buffer_load16(rs, lane_off);
        }
    }
}

// K tile from registers into LDS in format FMT.  kdst / ksdst: LDS addresses of the codes and of the scale bytes.
// PT: Alg. 2 Step 2: every key row is first multiplied by 2688 / rowmax; inv_sk[r] is that factor for chunk round r
// (the caller computes it once per tile for both formats, see key_token_scales).
// k_lane / s_lane: stage_k_lane / stage_s_lane of the thread.
template <typename C, int FMT, bool PT>
DMA_DEV void stage_k(const v4i (&reg)[C::CPT], unsigned kdst, unsigned ksdst, unsigned k_lane, unsigned s_lane,
                     const float (&inv_sk)[C::CPT], const float (&bam)[C::CPT])
{
    // bam[r] (PT): the largest magnitude of the lane's MX block in round r before the row is scaled; rounding is monotone,
    // so the block maximum of the scaled values is the scaled block maximum.
    constexpr int KPR = C::T / C::CPR;                       // keys per chunk round
    constexpr int STRIDE = C::template kstride<FMT>();
    const unsigned ka = pin(kdst + k_lane);
    const unsigned sa = pin(ksdst + s_lane);                  // every lane stores its block's scale: no divergence
#pragma unroll
    for (int r = 0; r < C::CPT; ++r) {
        if constexpr (FMT == FMT_BF16) {
            lds_write<v4i>(ka + r * KPR * STRIDE, reg[r]);
        } else if constexpr (FMT == FMT_E2M1 && !PT) {
            // keys are not pre-scaled: block maximum and converts work on the packed bf16 directly
            const int code = max((int)(quad_max_u32(amax8_bf16_bits(reg[r])) >> 7) - 2, 0);
            lds_write<int>(ka + r * KPR * STRIDE, encode8_e2m1_bf16(reg[r], code));
            lds_write<uint8_t>(sa + r * KPR * C::CPR, (uint8_t)code);
        } else if constexpr (FMT == FMT_E2M1) {
            float x[8];
            unpack8<false>(reg[r], 1.f, x);
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] = __fmul_rn(x[e], inv_sk[r]);
            const int code = e8m0_code<FMT_E2M1>(__fmul_rn(bam[r], inv_sk[r]));
            lds_write<int>(ka + r * KPR * STRIDE, encode8_e2m1(x, code));
            lds_write<uint8_t>(sa + r * KPR * C::CPR, (uint8_t)code);
        } else {
            float x[8];
            unpack8<false>(reg[r], 1.f, x);
            float amax;
            if constexpr (PT) {
#pragma unroll
                for (int e = 0; e < 8; ++e) x[e] = __fmul_rn(x[e], inv_sk[r]);
                amax = __fmul_rn(bam[r], inv_sk[r]);
            } else {
                amax = quad_max(amax8(x));
            }
            const int code = e8m0_code<FMT>(amax);
            if constexpr (FMT == FMT_E4M3_X || FMT == FMT_E5M2_X) {
                lds_write<v4i>(ka + r * KPR * STRIDE, quant_dequant8<FMT>(x, code));
            } else {
                lds_write<v2i>(ka + r * KPR * STRIDE, encode8_e4m3(x, code));
                lds_write<uint8_t>(sa + r * KPR * C::CPR, (uint8_t)code);
            }
        }
    }
}

// V tile from registers into LDS, 16-byte chunks swizzled (see Cfg::v_swizzle).
template <typename C>
DMA_DEV void stage_v(const v4i (&reg)[C::CPT], unsigned vdst, unsigned v_lane)
{
    constexpr int KPR = C::T / C::CPR;
    static_assert(KPR % 4 == 0, "swizzle of a row must not depend on the chunk round");
    const unsigned va = pin(vdst + v_lane);
#pragma unroll
    for (int r = 0; r < C::CPT; ++r) lds_write<v4i>(va + r * KPR * C::VS, reg[r]);
}

// V tile (thread mapping of vmx_thread) from registers into LDS as MXFP8-E4M3 with blocks of 32 keys per column: the
// wave's 32 keys of a column are spread over its chunk rounds and over the lanes that share lane % VCW.
template <typename C>
DMA_DEV void stage_v_mx(const v4i (&reg)[C::CPT], unsigned vdst, int tid)
{
    int kb, key, chunk;
    vmx_thread<C>(fresh(tid), kb, key, chunk);
    unsigned am[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        unsigned a = 0u;
#pragma unroll
        for (int r = 0; r < C::CPT; ++r) a = pk_max_u16(a, (unsigned)reg[r][t] & 0x7fff7fffu);
        am[t] = strided_lane_max_u16<C::VCW>(a);
    }
    // column t of the chunk: scale byte max(biased exponent - 8, 0) (Alg. 2 Steps 6-7 with e_max = 8) and 2^(127 - byte)
    int code[8];
    float inv[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        const int bits = (t & 1) ? (int)(am[t >> 1] >> 16) : (int)(am[t >> 1] & 0xffffu);
        code[t] = max((bits >> 7) - 8, 0);
        inv[t] = __int_as_float((254 - code[t]) << 23);
    }
    const unsigned va = pin(vdst + (32 * kb + key) * C::VS8 + chunk * 8);
#pragma unroll
    for (int r = 0; r < C::CPT; ++r) {
        float x[8];
        unpack8<false>(reg[r], 1.f, x);
        lds_write<v2i>(va + r * C::VRG * C::VS8, encode8_e4m3_each(x, inv));
    }
    if (key == 0) {
        v2i sc;
        sc[0] = code[0] | (code[1] << 8) | (code[2] << 16) | (code[3] << 24);
        sc[1] = code[4] | (code[5] << 8) | (code[6] << 16) | (code[7] << 24);
        lds_write<v2i>(vdst + C::V8CODES + kb * C::D + chunk * 8, sc);
    }
}

// The P^T operand of the value part for one wave and one key tile: bf16 pairs (16 keys per group), or, for the
// MX-format P V, E4M3 codes of 64 keys per group with the lane's scale byte.
template <typename C, bool PVMX>
struct PTile {
    v8bf b[2 * C::NKB];
};
template <typename C>
struct PTile<C, true> {
    v8i q[C::NKB / 2];
    int sc[C::NKB / 2];
};

// ---------------------------------------------------------------------------------------------
// One key tile for one wave: scores, mask, online softmax, P V
// ---------------------------------------------------------------------------------------------
template <int FMT, int H>
DMA_DEV v16f mfma_mx(const v8i& a, const v8i& b, const v16f& c, int sa, int sb)
{
    constexpr int code = (FMT == FMT_E2M1) ? 4 : 0;
    // sa: the K-side scale sits in byte 0 of its own dword; sb: byte H of the query scale dword
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, code, code, 0, sa, H, sb);
}

DMA_DEV v8i widen(const v4i& lo) { return v8i{lo[0], lo[1], lo[2], lo[3], 0, 0, 0, 0}; }
DMA_DEV v8i widen(const v4i& lo, const v4i& hi) { return v8i{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]}; }

// First half of a key tile for one wave (all of its VALU work): scores S^T, causal mask, new running maximum,
// rescale of l and O by 2^(m_old - m_new), probabilities P = 2^(S - m) summed into l and rounded to bf16.
// The result is P^T packed as the B operands of the value part: pb[grp] holds keys 16 grp .. 16 grp + 15.
// ksrc / kssrc: LDS addresses of the tile's K codes / scale bytes.
// MAYBE_DIAG = false compiles the mask away (tiles strictly below the diagonal).
// after_mfma() runs between the matrix part and the softmax part (the caller's global loads go there).
// PT (per-token scale, Alg. 2 Step 2): the product of the codes is multiplied by S_q of the query row (q_sq) and S_q of
// the key (one float per key at ktssrc) before the maximum is taken.
// PVMX (MX-format P V): the probabilities leave as MXFP8-E4M3 blocks of 32 keys.  The lane holds 16 keys of every
// 32-key block of its query (the other half-wave holds the other 16): keys 8 v + 4 g + b of block kb are byte b of
// VGPR v (block 2c) or 4 + v (block 2c + 1) of the operand of key group c, which is the order the V^T operand is read
// in (value_vmx_lane).  The block's scale comes from its largest probability 2^max(S - m): floor of that exponent.
template <typename C, int FMT, bool MAYBE_DIAG, bool PT, bool PVMX, int QR, typename F>
DMA_DEV void score_part(const v4i (&qr)[QR], int qscale, unsigned ksrc, unsigned kssrc, unsigned k_lane, unsigned s_lane,
                        unsigned ktssrc, float q_sq, bool diagonal, int key_limit, int qrow_in_tile, int lane, float c,
                        float& m, float& mfloor, float& l, v16f (&o)[C::NDB], PTile<C, PVMX>& pt, F&& after_mfma)
{
    lane = fresh(lane);
    const int j = lane & 31, g = lane >> 5;
    v16f s[C::NKB];
    constexpr int STRIDE = C::template kstride<FMT>();
    const unsigned ka = pin(ksrc + k_lane);                       // the lane's key row of 32-key block 0 (score_k_lane)
    // The accumulators start at -m (the running maximum so far), so the products arrive as S - m and the
    // subtraction of the maximum costs nothing in the common case of a maximum that does not move.
    // (One register tuple holds the start value; the first MFMA of every 32-key block reads it as its C operand.)
    constexpr bool SCALE_AFTER = PT && FMT != FMT_BF16;       // the score is rescaled after the product
    const float acc0 = (FMT == FMT_BF16 || SCALE_AFTER) ? 0.f : -m;
    const v16f sinit = {acc0, acc0, acc0, acc0, acc0, acc0, acc0, acc0, acc0, acc0, acc0, acc0, acc0, acc0, acc0, acc0};

    // ---- S^T = K . Q^T.  Operands are fetched from LDS ahead of the MFMAs that use them.
    if constexpr (FMT == FMT_E2M1) {
        // operands of two 32-key blocks at a time (2 * NH 16-byte reads + 2 scale dwords) ahead of their MFMAs,
        // which go h-major so that the two MFMAs into one accumulator are not adjacent
        // scale of MX block 2h + g of the lane's key: byte 0 of the dword at chunk 4 (2h + g) of the key's scale row
        const unsigned sa = pin(kssrc + s_lane);
        static_assert(C::NKB % 2 == 0, "key tile must hold an even number of 32-key blocks");
        v4i a[2][2][C::NH];
        int ksc[2][2][C::NH];
        auto fetch = [&](int pair) {
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int kb = 2 * pair + u;
#pragma unroll
                for (int h = 0; h < C::NH; ++h) {
                    ksc[pair & 1][u][h] = lds_read<int>(sa + kb * 32 * C::CPR + 8 * h);
                    a[pair & 1][u][h] = lds_read<v4i>(ka + kb * 32 * STRIDE + 32 * h);
                }
            }
        };
        fetch(0);
#pragma unroll
        for (int pair = 0; pair < C::NKB / 2; ++pair) {
            if (pair + 1 < C::NKB / 2) fetch(pair + 1);
            static_for<C::NH>([&](auto H) {
                constexpr int h = H;
                const v8i b = widen(qr[h]);
#pragma unroll
                for (int u = 0; u < 2; ++u)
                    s[2 * pair + u] = mfma_mx<FMT, h>(widen(a[pair & 1][u][h]), b, h == 0 ? sinit : s[2 * pair + u], ksc[pair & 1][u][h], qscale);
            });
            __builtin_amdgcn_sched_barrier(0);
        }
    } else if constexpr (FMT == FMT_E4M3) {
        const unsigned sa = pin(kssrc + s_lane);
#pragma unroll
        for (int kb = 0; kb < C::NKB; ++kb) {
            static_for<C::NH>([&](auto H) {
                constexpr int h = H;
                const int ksc = lds_read<int>(sa + kb * 32 * C::CPR + 8 * h);
                const v4i lo = lds_read<v4i>(ka + kb * 32 * STRIDE + 64 * h);
                const v4i hi = lds_read<v4i>(ka + kb * 32 * STRIDE + 64 * h + 32);
                s[kb] = mfma_mx<FMT, h>(widen(lo, hi), widen(qr[2 * h], qr[2 * h + 1]), h == 0 ? sinit : s[kb], ksc, qscale);
            });
        }
    } else {
        // bf16 MFMA (unquantized, or MXFP8 decoded exactly): NKK k=16 steps per 32-key block, in units of UK steps;
        // the next unit's operands are in flight while the current unit multiplies.  Step kk = 4h + t multiplies the
        // lane's chunk t of MX block 2h + g (see load_q_raw): byte 128 h + 64 g + 16 t of the key's bf16 row.
        constexpr int UK = 4, UPB = C::NKK / UK, NU = C::NKB * UPB;
        static_assert(C::NKK % UK == 0, "head dimension must be a multiple of 64");
        v4i a[2][UK];
        auto fetch = [&](int u) {
#pragma unroll
            for (int i = 0; i < UK; ++i)
                a[u & 1][i] = lds_read<v4i>(ka + (u / UPB) * 32 * STRIDE + 16 * ((u % UPB) * UK + i) + 64 * (((u % UPB) * UK + i) / 4));
        };
        fetch(0);
#pragma unroll
        for (int u = 0; u < NU; ++u) {
            if (u + 1 < NU) fetch(u + 1);
            const int kb = u / UPB;
#pragma unroll
            for (int i = 0; i < UK; ++i)
                s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a[u & 1][i]),
                                                                __builtin_bit_cast(v8bf, qr[(u % UPB) * UK + i]),
                                                                (u % UPB == 0 && i == 0) ? sinit : s[kb], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (FMT == FMT_BF16) {                 // unquantized operands: the softmax factor multiplies the score
#pragma unroll
            for (int kb = 0; kb < C::NKB; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) s[kb][r] = __builtin_fmaf(s[kb][r], c, -m);
        }
    }

    if constexpr (SCALE_AFTER) {
        // register r of 32-key block kb is key 32 kb + 8 (r / 4) + 4 g + r % 4: four consecutive scales per read
        const unsigned ta = pin(ktssrc + 16 * g);
#pragma unroll
        for (int kb = 0; kb < C::NKB; ++kb)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                const v4f sk = lds_read<v4f>(ta + 4 * (32 * kb + 8 * r4));
#pragma unroll
                for (int e = 0; e < 4; ++e) s[kb][4 * r4 + e] = __builtin_fmaf(s[kb][4 * r4 + e], q_sq * sk[e], -m);
            }
    }
    after_mfma();

    // ---- causal mask on the tile that straddles the diagonal (key > query -> -inf) and / or the keys of a partial
    // last tile that lie past the end of the sequence (key >= key_limit -> -inf)
    if constexpr (MAYBE_DIAG) {
        if (diagonal || key_limit < C::BT) {
            const int last_key = min(diagonal ? qrow_in_tile + j : C::BT - 1, key_limit - 1);
#pragma unroll
            for (int kb = 0; kb < C::NKB; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int kj = kb * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
                    if (kj > last_key) s[kb][r] = -INFINITY;
                }
        }
    }

    // ---- online softmax in base 2.  s holds S - m.  delta = how far the row maximum moves (>= 0; on the first tile
    // of a row, where m is only the arbitrary start value 0, any sign: mfloor is -inf there and 0 afterwards).
    float mx = -INFINITY;
    float bmax[C::NKB];                                   // MX-format P V: maxima per 32-key block
    if constexpr (PVMX) {
#pragma unroll
        for (int kb = 0; kb < C::NKB; ++kb) {
            bmax[kb] = -INFINITY;
#pragma unroll
            for (int r = 0; r < 16; ++r) bmax[kb] = fmaxf(bmax[kb], s[kb][r]);
            bmax[kb] = cross_half_max(bmax[kb]);
            mx = fmaxf(mx, bmax[kb]);
        }
    } else {
#pragma unroll
        for (int kb = 0; kb < C::NKB; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kb][r]);
        mx = cross_half_max(mx);
    }
    const float delta = fmaxf(mx, mfloor);
    const float mnew = m + delta;
    const float alpha = __builtin_amdgcn_exp2f(fminf(m - mnew, 0.f));     // first tile: l and O are 0, any finite factor does
    m = mnew;
    mfloor = 0.f;
    if (__builtin_amdgcn_ballot_w64(delta != 0.0f) != 0) {      // skipped when no row of the wave moved its maximum
#pragma unroll
        for (int db = 0; db < C::NDB; ++db) o[db] *= alpha;
#pragma unroll
        for (int kb = 0; kb < C::NKB; ++kb) s[kb] -= delta;
    }

    // ---- P = 2^(S - m): row sums from the binary32 values; for the P V product bf16 (round to nearest even), or ...
    float psum[2] = {0.f, 0.f};
    if constexpr (!PVMX) {
#pragma unroll
        for (int grp = 0; grp < 2 * C::NKB; ++grp) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const float p0 = __builtin_amdgcn_exp2f(s[grp >> 1][8 * (grp & 1) + 2 * t]);
                const float p1 = __builtin_amdgcn_exp2f(s[grp >> 1][8 * (grp & 1) + 2 * t + 1]);
                psum[0] += p0;
                psum[1] += p1;
                const v2bf h2 = __builtin_convertvector(v2f{p0, p1}, v2bf);
                pt.b[grp][2 * t] = h2[0];
                pt.b[grp][2 * t + 1] = h2[1];
            }
        }
    } else {
        // ... MXFP8-E4M3 blocks of 32 keys.  The block maximum of S - m after the rescale is bmax - delta (rounding is
        // monotone); the largest probability of the block is 2^that, so its biased exponent is 127 + floor(that) and the
        // scale byte max(127 + floor - 8, 0).  A block with every key masked has maximum -inf and scale byte 0.
#pragma unroll
        for (int cgrp = 0; cgrp < C::NKB / 2; ++cgrp) {
            int code[2];
            int packed[8];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int kb = 2 * cgrp + u;
                const float top = fmaxf(bmax[kb] - delta, -256.f);
                code[u] = max((int)__builtin_floorf(top) + 119, 0);
#pragma unroll
                for (int h8 = 0; h8 < 2; ++h8) {
                    float p[8];
#pragma unroll
                    for (int t = 0; t < 8; ++t) {
                        p[t] = __builtin_amdgcn_exp2f(s[kb][8 * h8 + t]);
                        psum[t & 1] += p[t];
                    }
                    const v2i e = encode8_e4m3_prob(p, code[u]);
                    packed[4 * u + 2 * h8] = e[0];
                    packed[4 * u + 2 * h8 + 1] = e[1];
                }
            }
            pt.q[cgrp] = v8i{packed[0], packed[1], packed[2], packed[3], packed[4], packed[5], packed[6], packed[7]};
            pt.sc[cgrp] = g ? code[1] : code[0];
        }
    }
    l = l * alpha + (psum[0] + psum[1]);
}

// Second half (all matrix work): O^T += V^T . P^T in groups of 16 keys; the V^T operands of the next group are in
// flight from LDS while the MFMAs of the current group run.  vsrc: LDS address of the V tile.
template <typename C>
DMA_DEV void value_part(unsigned vsrc, const unsigned (&v_lane)[C::NDB], v16f (&o)[C::NDB], const PTile<C, false>& pt)
{
    const v8bf (&pb)[2 * C::NKB] = pt.b;
    // va[db]: the lane's address for d-block db in the tile's first patch (value_v_lane); other patches are constant offsets
    unsigned va[C::NDB];
#pragma unroll
    for (int db = 0; db < C::NDB; ++db) va[db] = pin(vsrc + v_lane[db]);

    auto read_vt = [&](v8s (&a)[C::NDB], int grp) {             // V^T operands of key group grp (16 keys)
#pragma unroll
        for (int db = 0; db < C::NDB; ++db) {
            const v4s a0 = lds_read_tr16(va[db] + grp * 16 * C::VS);
            const v4s a1 = lds_read_tr16(va[db] + grp * 16 * C::VS + 8 * C::VS);
            a[db] = v8s{a0[0], a0[1], a0[2], a0[3], a1[0], a1[1], a1[2], a1[3]};
        }
    };
    constexpr int NG = 2 * C::NKB;
    v8s vt[3][C::NDB];                       // operands of groups grp, grp+1 and grp+2 in rotation
    read_vt(vt[0], 0);
    if (NG > 1) read_vt(vt[1], 1);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int grp = 0; grp < NG; ++grp) {
        if (grp + 2 < NG) read_vt(vt[(grp + 2) % 3], grp + 2);
#pragma unroll
        for (int db = 0; db < C::NDB; ++db)
            o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, vt[grp % 3][db]), pb[grp], o[db], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// The same for the MX-format P V: O^T += V^T . P^T on the block-scaled FP8 MFMA in groups of 64 keys.  vsrc: LDS
// address of the E4M3 V tile (codes, then the scale bytes [32-key block][column]).
template <typename C>
DMA_DEV void value_part(unsigned vsrc, int lane, v16f (&o)[C::NDB], const PTile<C, true>& pt)
{
    lane = fresh(lane);
    const unsigned va = pin(vsrc + value_vmx_lane<C>(lane));
    const unsigned sa = pin(vsrc + C::V8CODES + (lane >> 5) * C::D + (lane & 31));
#pragma unroll
    for (int cgrp = 0; cgrp < C::NKB / 2; ++cgrp) {
        v8i a[C::NDB];
        int vsc[C::NDB];
#pragma unroll
        for (int db = 0; db < C::NDB; ++db) {
            vsc[db] = (int)lds_read<uint8_t>(sa + 2 * cgrp * C::D + 32 * db);
            int w[8];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const v2i t = lds_read_tr8(va + (64 * cgrp + 16 * r) * C::VS8 + 32 * db);
                w[2 * r] = t[0];
                w[2 * r + 1] = t[1];
            }
            a[db] = v8i{w[0], w[1], w[2], w[3], w[4], w[5], w[6], w[7]};
        }
#pragma unroll
        for (int db = 0; db < C::NDB; ++db)
            o[db] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[db], pt.q[cgrp], o[db], 0, 0, 0, vsc[db], 0, pt.sc[cgrp]);
    }
}

// ---------------------------------------------------------------------------------------------
// The kernel
// ---------------------------------------------------------------------------------------------
// Alg. 2 Step 2 for the keys of a tile: per chunk round the row maximum over the CPR lanes of the row, S_q into LDS
// (one float per key at ktsdst), 1 / S_q returned for the quantization (inv_sk), and with it the largest magnitude of
// the lane's MX block before the scaling (bam), from which stage_k gets the block's shared scale without a second pass.
// kam / given: the maximum of the group each key row belongs to, when the caller supplies group maxima (a coarser
// granularity than the row) instead of the row's own maximum.
// The two divisions of a row's scale are the expensive part and every lane of a row would repeat them: the lanes of a
// quad take one chunk round each instead (lane q of the quad: round base + q), divide once, and hand the reciprocal to
// the other three with a quad broadcast.
template <typename C>
DMA_DEV void key_token_scales(const v4i (&reg)[C::CPT], float (&inv_sk)[C::CPT], float (&bam)[C::CPT], unsigned ktsdst, int tid,
                              const float (&kam)[C::CPT], bool given)
{
    constexpr int KPR = C::T / C::CPR;
    static_assert(C::CPR % 4 == 0, "a quad of lanes lies inside one key row");
    tid = fresh(tid);
    const int key0 = tid / C::CPR, dc = tid % C::CPR, ql = tid & 3;
    float am[C::CPT];
#pragma unroll
    for (int r = 0; r < C::CPT; ++r) {
        float x[8];
        unpack8<false>(reg[r], 1.f, x);
        bam[r] = quad_max(amax8(x));                     // the lane's MX block (a quad of lanes), for stage_k
        float row = bam[r];                              // ... and on to the whole row: group_max's remaining steps
        if constexpr (C::CPR >= 8) row = fmaxf(row, __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(row), 0x141, 0xF, 0xF, true)));
        if constexpr (C::CPR >= 16) row = fmaxf(row, __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(row), 0x140, 0xF, 0xF, true)));
        am[r] = given ? kam[r] : row;
    }
#pragma unroll
    for (int base = 0; base < C::CPT; base += 4) {
        float mine = am[base];
#pragma unroll
        for (int j = 1; j < 4; ++j)
            if (base + j < C::CPT) mine = (ql == j) ? am[base + j] : mine;
        float sk, inv;
        token_scale(mine, sk, inv);
        const int invb = __float_as_int(inv);
        if (base + 0 < C::CPT) inv_sk[base + 0] = __int_as_float(__builtin_amdgcn_mov_dpp(invb, 0x00, 0xF, 0xF, true));
        if (base + 1 < C::CPT) inv_sk[base + 1] = __int_as_float(__builtin_amdgcn_mov_dpp(invb, 0x55, 0xF, 0xF, true));
        if (base + 2 < C::CPT) inv_sk[base + 2] = __int_as_float(__builtin_amdgcn_mov_dpp(invb, 0xAA, 0xF, 0xF, true));
        if (base + 3 < C::CPT) inv_sk[base + 3] = __int_as_float(__builtin_amdgcn_mov_dpp(invb, 0xFF, 0xF, 0xF, true));
        // S_q of round base + q goes to LDS from lane q of the row's first quad
        if (dc < 4 && base + dc < C::CPT) lds_write<float>(ktsdst + 4 * (key0 + (base + dc) * KPR), sk);
    }
}

// The group maxima of the key rows of a tile, one per chunk round of the thread (rows >= S: 0).
template <typename C>
DMA_DEV void load_key_amax(float (&kam)[C::CPT], const float* __restrict__ amax_head, int row0, int S, int tid)
{
    constexpr int KPR = C::T / C::CPR;
    const int key0 = row0 + fresh(tid) / C::CPR;
#pragma unroll
    for (int r = 0; r < C::CPT; ++r) kam[r] = (key0 + r * KPR < S) ? amax_head[key0 + r * KPR] : 0.f;
}

// K and V of one key tile from registers into LDS: K in the low format if some wave computes the tile in Phase 1,
// in the high format if some wave computes it in Phase 2.
template <typename C, int LO, int HI, bool PT, bool PVMX>
DMA_DEV void stage_tile(const v4i (&kreg)[C::CPT], const v4i (&vreg)[C::CPT], bool any_lo, bool any_hi,
                        unsigned klo, unsigned kslo, unsigned khi, unsigned kshi, unsigned kts, unsigned vdst,
                        const LaneOffsets<C, LO>& lo, int tid, const float (&kam)[C::CPT], bool kam_given)
{
    float inv_sk[C::CPT], bam[C::CPT];
#pragma unroll
    for (int r = 0; r < C::CPT; ++r) inv_sk[r] = 1.f, bam[r] = 0.f;
    if constexpr (PT) key_token_scales<C>(kreg, inv_sk, bam, kts, tid, kam, kam_given);
    if (any_lo) stage_k<C, LO, PT>(kreg, klo, kslo, lo.stage_k, lo.stage_s, inv_sk, bam);
    if constexpr (LO != HI) {
        if (any_hi) stage_k<C, HI, PT>(kreg, khi, kshi, stage_k_lane<C, HI>(fresh(tid)), lo.stage_s, inv_sk, bam);
    }
    if constexpr (PVMX) stage_v_mx<C>(vreg, vdst, tid);
    else stage_v<C>(vreg, vdst, lo.stage_v);
}

// GENERAL = false: Alg. 1 as printed (causal, no sink window; sink_arg / causal_arg are ignored): main tiles then band
// tiles, two loops in a row.  GENERAL = true: sink window and / or no causal mask: runs of main and band tiles alternate.
// PT: per-token scale of Alg. 2 Step 2 on queries and keys (built with GENERAL only).
// PVMX: the P V product in MXFP8-E4M3 with blocks of 32 keys (an extension beyond Alg. 1, which keeps P and V in 16 bit).
template <int D, int BT, int TPW, int LO, int HI, bool GENERAL, bool PT, bool PVMX>
__global__ void __launch_bounds__((BT / 32) * TPW * 64, 2)
dma_attn_fwd_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                    const uint16_t* __restrict__ v, float* __restrict__ out,
                    int B, int Hq, int Hkv, int S, int band, int sink_arg, int causal_arg, float c, int head_block,
                    const float* __restrict__ q_amax, const float* __restrict__ k_amax)
{
    // q_amax / k_amax (PT only, both or neither): group maxima per query row [B, Hq, S] / key row [B, Hkv, S] that replace
    // the rows' own maxima in Alg. 2 Step 2 (a coarser granularity of the scale); null: per-token.
    const bool amax_given = PT && q_amax != nullptr;
    const int sink = GENERAL ? sink_arg : 0;
    const bool causal = GENERAL ? (causal_arg != 0) : true;
    using C = Cfg<D, BT, TPW>;
    constexpr bool TWO = (LO != HI);
    constexpr int KLO = C::template kbytes<LO>();
    constexpr int KHI = TWO ? C::template kbytes<HI>() : 0;
    constexpr int QRLO = C::template qregs<LO>();
    constexpr int QRHI = TWO ? C::template qregs<HI>() : 1;
    // LDS map (bytes): V, the low-format K and the high-format K (each + scale bytes) double-buffered for the pipelined
    // tile loops.  The output transpose of the epilogue reuses the same memory.
    constexpr int OFF_V = 0;
    constexpr int VB = PVMX ? C::V8BYTES : C::VBYTES;
    constexpr int OFF_KLO = OFF_V + 2 * VB;
    constexpr int OFF_KSLO = OFF_KLO + 2 * KLO;
    constexpr int OFF_KHI = OFF_KSLO + 2 * C::KSC;
    constexpr bool HI_SCALES = TWO && !uses_bf16_mfma(HI);   // the decoded-to-bf16 high format carries no scale bytes
    constexpr int OFF_KSHI = OFF_KHI + 2 * KHI;
    constexpr int EPI_COLS = 64;                         // output columns per epilogue pass
    constexpr int EPI_STRIDE = EPI_COLS * 4 + 16;        // bytes per staged output row (padded against bank conflicts)
    constexpr int EPI_WAVE = 32 * EPI_STRIDE;
    constexpr int OFF_KTS = OFF_KSHI + (HI_SCALES ? 2 * C::KSC : 0);      // per-token key scales: one float per key
    constexpr int LDS_TOTAL = cmax<OFF_KTS + (PT ? 2 * BT * 4 : 0), C::NW * EPI_WAVE>();
    static_assert(LDS_TOTAL <= 160 * 1024, "LDS budget of one CU");
    static_assert(D % EPI_COLS == 0, "epilogue works on 64-column slabs");
    __shared__ __attribute__((aligned(16))) uint8_t lds[LDS_TOTAL];
    const unsigned lds0 = (unsigned)(uintptr_t)(DMA_LDS uint8_t*)lds;
    auto v_at = [&](int buf) { return lds0 + OFF_V + buf * VB; };
    auto klo_at = [&](int buf) { return lds0 + OFF_KLO + buf * KLO; };
    auto kslo_at = [&](int buf) { return lds0 + OFF_KSLO + buf * C::KSC; };
    auto khi_at = [&](int buf) { return lds0 + OFF_KHI + buf * KHI; };
    auto kshi_at = [&](int buf) { return lds0 + OFF_KSHI + (HI_SCALES ? buf * C::KSC : 0); };
    auto kts_at = [&](int buf) { return lds0 + OFF_KTS + (PT ? buf * BT * 4 : 0); };
    auto load_v = [&](v4i (&reg)[C::CPT], const uint16_t* mat, int row0, int S_, int tid_) __attribute__((always_inline)) {
        if constexpr (PVMX) load_tile_vmx<C, GENERAL>(reg, mat, row0, S_, tid_);
        else load_tile<C, GENERAL>(reg, mat, row0, S_, tid_);
    };
    auto pv = [&](unsigned vsrc, const LaneOffsets<C, LO>& lo_, int lane_, v16f (&o_)[C::NDB], const PTile<C, PVMX>& p_) __attribute__((always_inline)) {
        if constexpr (PVMX) value_part<C>(vsrc, lane_, o_, p_);
        else value_part<C>(vsrc, lo_.value_v, o_, p_);
    };

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    LaneOffsets<C, LO> lofs;
    lofs.init(tid, lane);

    // ---- static schedule.  The grid is one workgroup per CU; a work item is (batch, query head, group of TPW query
    // tiles) and costs about 2 * grp + 2 key-tile steps.  Items are ranked heaviest first within blocks of
    // `head_block` query heads and dealt to the workgroups in boustrophedon order (round 0: worker 0, 1, ..., W-1;
    // round 1: W-1, ..., 0; ...), which gives every worker the same load to within the lightest items, without
    // atomics and whatever order the hardware starts workgroups in; a block is an even number of rounds (or
    // everything), so the workers move from block to block together and share few K/V streams at a time.  When the
    // (batch, kv head) units divide over the 8 XCDs (workgroup i runs on XCD i % 8), each XCD keeps its own units, so
    // the K/V stream of a unit stays in one L2.
    // Logical tiles per sequence; the last one may be partial.  When N is not a multiple of TPW (GENERAL instances only)
    // the last group is filled up with query tiles that lie wholly past the end of the sequence: their rows load as
    // zeros, their stores are dropped by the bounds of the output's buffer resource, and under the causal mask they
    // alone visit key tile N, which loads as zeros too.  They cost one extra step in one item per head.
    const int N = (S + BT - 1) / BT;
    const int NG = (N + TPW - 1) / TPW;  // tile groups
    const int group = Hq / Hkv;
    const int units = B * Hkv;
    const bool by_xcd = (units % 8 == 0) && (gridDim.x % 8 == 0);
    const int xcd = by_xcd ? (int)(blockIdx.x & 7) : 0;
    const int slot = by_xcd ? (int)(blockIdx.x >> 3) : (int)blockIdx.x;
    const int workers = by_xcd ? (int)(gridDim.x >> 3) : (int)gridDim.x;
    const int heads_x = by_xcd ? (units / 8) * group : B * Hq;       // query heads ranked together
    const int items = heads_x * NG;

    for (int round = 0;; ++round) {
        const int pos = round * workers + ((round & 1) ? workers - 1 - slot : slot);
        if (pos >= items) break;
        const int blk = pos / (head_block * NG), within = pos % (head_block * NG);
        const int grp = NG - 1 - within / head_block;
        const int hx = blk * head_block + within % head_block;
        const int unit = by_xcd ? (hx / group) * 8 + xcd : hx / group;
        const int b = unit / Hkv;
        const int hkv = unit % Hkv;
        const int hq = hkv * group + hx % group;
        const uint16_t* qhead = q + ((int64_t)b * Hq + hq) * S * D;
        const uint16_t* khead = k + ((int64_t)b * Hkv + hkv) * S * D;
        const uint16_t* vhead = v + ((int64_t)b * Hkv + hkv) * S * D;
        float* ohead = out + ((int64_t)b * Hq + hq) * S * D;
        const float* qam_head = amax_given ? q_amax + ((int64_t)b * Hq + hq) * S : nullptr;
        const float* kam_head = amax_given ? k_amax + ((int64_t)b * Hkv + hkv) * S : nullptr;

        // ---- this wave's logical tile and the precision rule (Alg. 1: for query tile `it`, key tile jt is high
        // precision iff it lies in the diagonal window, it - jt < band; extensions: the first `sink` key tiles are high
        // precision for every query tile, and without the causal mask every key tile is visited and the window is
        // |it - jt| < band).  Key tiles are visited in ascending order.
        const int it0 = grp * TPW, last = it0 + TPW - 1;
        const int it = it0 + wave / C::WPT;
        const int qrow_in_tile = (wave % C::WPT) * 32;
        const int qrow = it * BT + qrow_in_tile;
        const int nt = causal ? last + 1 : N;            // this item visits key tiles [0, nt)
        auto tile_hi = [&](int qt, int jt) __attribute__((always_inline)) {             // does query tile qt compute key tile jt in the high format?
            if (!TWO) return false;
            if (jt < sink) return true;
            const int dist = (causal || qt >= jt) ? qt - jt : jt - qt;
            return dist < band;
        };
        // Key tiles split into "main" tiles -- low format, unmasked and computed by every wave of the workgroup --
        // and "band" tiles, where waves differ (skipped past the wave's diagonal, Phase 1 or Phase 2, masked on the
        // wave's diagonal tile): band tiles are [0, s1) (the sink) and [w0, w1) (around the diagonal).
        int w0, w1, s1 = TWO ? min(sink, nt) : 0;
        if (causal) {
            w0 = (TWO && band > 0) ? max(0, it0 + 1 - band) : it0;
            w1 = nt;
        } else if (TWO && band > 0) {
            w0 = max(0, it0 + 1 - band);
            w1 = min(N, last + band);
        } else {
            w0 = w1 = nt;
        }
        // without the causal mask a partial last tile must be a band tile (its missing keys are masked there)
        const bool ragged_tail = !causal && S % BT != 0;
        if (ragged_tail) w0 = min(w0, nt - 1);
        if (s1 > w0) { w1 = max(w1, s1); w0 = 0; s1 = 0; }
        // what the workgroup needs of key tile jt in LDS
        auto needs = [&](int jt, bool& any_lo, bool& any_hi) __attribute__((always_inline)) {
            any_lo = !TWO;
            any_hi = false;
            if constexpr (TWO) {
#pragma unroll
                for (int w = 0; w < TPW; ++w) {
                    if (causal && jt > it0 + w) continue;
                    const bool h = tile_hi(it0 + w, jt);
                    any_hi |= h;
                    any_lo |= !h;
                }
            }
        };

        // Running maximum m and sum l (Alg. 1 starts m at -inf and l at 1, and the first rescale factor 2^(-inf) erases
        // that l).  Here m starts at 0 with l = 0 and mfloor = -inf marks "no tile seen yet": the first tile then sets m to
        // its row maximum whatever the sign, which gives the same m, l and O as Alg. 1 after that tile.
        float m = 0.f, mfloor = -INFINITY, l = 0.f;
        v16f o[C::NDB];
#pragma unroll
        for (int db = 0; db < C::NDB; ++db) o[db] = v16f{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};

        // ---- prologue: key tile 0 and the query operands (all loads in flight together), tile 0 into LDS buffer 0.
        // Invariant from here on: the K/V registers hold the tile after the one staged last, if there is one.
        v4i kreg[C::CPT], vreg[C::CPT];
        float kam[C::CPT];                               // group maxima of the key rows in kreg (when given)
#pragma unroll
        for (int r = 0; r < C::CPT; ++r) kam[r] = 0.f;
        auto load_k = [&](int jt) __attribute__((always_inline)) {                   // K tile jt (and its group maxima) into the registers
            load_tile<C, GENERAL>(kreg, khead, jt * BT, S, tid);
            if constexpr (PT) {
                if (amax_given) load_key_amax<C>(kam, kam_head, jt * BT, S, tid);
            }
        };
        PTile<C, PVMX> pb;
        v4i qr_lo[QRLO], qr_hi[QRHI];
        int qs_lo = 0, qs_hi = 0;
        float q_sq = 1.f;                                // S_q of the lane's query row (per-token scale)
        {
            v4i qraw[C::NKK];
            load_q_raw<C>(qraw, make_rsrc(qhead, (uint32_t)S * (D * 2)), qrow, fresh(lane) & 31, fresh(lane) >> 5);
            load_k(0);
            load_v(vreg, vhead, 0, S, tid);
            __builtin_amdgcn_sched_barrier(0);           // every request is out before the first result is needed
            float inv_sq = 1.f;
            if constexpr (PT) {
                float amax;
                if (amax_given) {
                    const int row = qrow + (fresh(lane) & 31);
                    amax = row < S ? qam_head[row] : 0.f;
                } else {
                    amax = q_row_amax<C>(qraw, c);
                }
                token_scale(amax, q_sq, inv_sq);
            }
            make_q<C, LO, PT>(qr_lo, qs_lo, qraw, c, inv_sq);
            if constexpr (TWO) {
                if (band > 0 || sink > 0) make_q<C, HI, PT>(qr_hi, qs_hi, qraw, c, inv_sq);
            }
        }
        auto stage_next = [&](int jt, int buf) __attribute__((always_inline)) {         // tile jt from the K/V registers into LDS buffer buf
            bool any_lo, any_hi;
            needs(jt, any_lo, any_hi);
            stage_tile<C, LO, HI, PT, PVMX>(kreg, vreg, any_lo, any_hi, klo_at(buf), kslo_at(buf), khi_at(buf), kshi_at(buf), kts_at(buf),
                                      v_at(buf), lofs, tid, kam, amax_given);
        };
        stage_next(0, 0);
        if (1 < nt) {
            load_k(1);
            load_v(vreg, vhead, BT, S, tid);
        }
        __syncthreads();

        // ---- tile loop.  Tile jt lives in LDS buffer jt & 1; one barrier per tile.  At the top of step jt the K and
        // V tiles jt+1 (loaded into registers during step jt-1) go into the other buffer (K quantized on the way) and
        // the loads of tile jt+2 start; then the wave computes tile jt.
        // (Direct global-to-LDS loads are not used for V: generated from the builtin, the compiler orders every later LDS
        // access behind them with a full vmcnt(0) wait, which exposes the memory latency; issued from inline assembly
        // they work, but the forward was measured 8 % slower than with V going through registers.)
        // On main tiles K of tile jt+2 is requested in the middle of the score part (after its MFMAs), V after it:
        // the two bursts of requests (every wave of the workgroup issues them at about the same point) are half as
        // long, and the matrix part of the score has 32 registers more.
        auto main_step = [&](int jt) __attribute__((always_inline)) {
            const int buf = jt & 1;
            if constexpr (!GENERAL && !PT && !PVMX) {
                // Alg. 1 as printed: a main tile is followed by at least two more tiles, so nothing here needs a
                // condition on jt.  The two waves of a SIMD (w and w + 4) take the staging of the next tile and their
                // score MFMAs in opposite order: the matrix pipe serves one wave at a time, the lower-numbered one
                // first, so wave w multiplies while wave w + 4 quantizes and stages, then the other way round, instead
                // of both staging and then one waiting for the other's MFMAs (measured -0.8 % on the 32k workload,
                // -0.5 % on the 8k prefill; the opposite assignment gains nothing).
                const bool mfma_first = C::NW == 8 && __builtin_amdgcn_readfirstlane(tid) < 256;
                if (!mfma_first) stage_next(jt + 1, buf ^ 1);
                score_part<C, LO, false, PT, PVMX>(qr_lo, qs_lo, klo_at(buf), kslo_at(buf), lofs.score_k, lofs.score_s, kts_at(buf), q_sq, false, BT, qrow_in_tile, lane, c, m, mfloor, l, o, pb,
                                         [&]() __attribute__((always_inline)) {
                                             if (mfma_first) stage_next(jt + 1, buf ^ 1);
                                             __builtin_amdgcn_sched_barrier(0);
                                             load_k(jt + 2);
                                         });
                load_v(vreg, vhead, (jt + 2) * BT, S, tid);
            } else {
                if (jt + 1 < nt) stage_next(jt + 1, buf ^ 1);
                score_part<C, LO, false, PT, PVMX>(qr_lo, qs_lo, klo_at(buf), kslo_at(buf), lofs.score_k, lofs.score_s, kts_at(buf), q_sq, false, BT, qrow_in_tile, lane, c, m, mfloor, l, o, pb,
                                         [&]() __attribute__((always_inline)) { if (jt + 2 < nt) load_k(jt + 2); });
                if (jt + 2 < nt) load_v(vreg, vhead, (jt + 2) * BT, S, tid);
            }
            pv(v_at(buf), lofs, lane, o, pb);
            __syncthreads();
        };
        auto band_step = [&](int jt) __attribute__((always_inline)) {
            const int buf = jt & 1;
            const bool active = !causal || jt <= it;
            const bool diagonal = causal && jt == it;
            // keys of this tile that exist (a partial last tile; under the causal mask the diagonal rule covers it)
            const int key_limit = causal ? BT : min(BT, S - jt * BT);
            if (jt + 1 < nt) stage_next(jt + 1, buf ^ 1);
            if (active) {
                if (!tile_hi(it, jt)) {
                    score_part<C, LO, true, PT, PVMX>(qr_lo, qs_lo, klo_at(buf), kslo_at(buf), lofs.score_k, lofs.score_s, kts_at(buf), q_sq, diagonal, key_limit, qrow_in_tile, lane, c, m, mfloor, l, o, pb, [] {});
                } else if constexpr (TWO) {
                    score_part<C, HI, true, PT, PVMX>(qr_hi, qs_hi, khi_at(buf), kshi_at(buf), score_k_lane<C, HI>(fresh(lane)), lofs.score_s, kts_at(buf), q_sq, diagonal, key_limit, qrow_in_tile, lane, c, m, mfloor, l, o, pb, [] {});
                }
            }
            if (jt + 2 < nt) {
                load_k(jt + 2);
                load_v(vreg, vhead, (jt + 2) * BT, S, tid);
            }
            if (active) pv(v_at(buf), lofs, lane, o, pb);
            __syncthreads();
        };
        if constexpr (!GENERAL) {
            for (int jt = 0; jt < w0; ++jt) main_step(jt);
            for (int jt = w0; jt < nt; ++jt) band_step(jt);
        } else {
            // four runs in a row (each may be empty): sink band tiles, main tiles, band tiles around the diagonal, and
            // (without the causal mask) the main tiles above the window
            // ... and a partial last tile, whose missing keys a band step masks
            const int mend = ragged_tail ? max(w1, nt - 1) : nt;
            for (int jt = 0; jt < s1; ++jt) band_step(jt);
            for (int jt = s1; jt < w0; ++jt) main_step(jt);
            for (int jt = w0; jt < w1; ++jt) band_step(jt);
            for (int jt = w1; jt < mend; ++jt) main_step(jt);
            for (int jt = mend; jt < nt; ++jt) band_step(jt);
        }

        // ---- O / l, transposed through LDS (free after the barrier above) so that every output row leaves as whole
        // 256-byte runs: the wave parks a 32 x 64 slab of its rows in its own LDS region and reads it back row-major,
        // four rows (16 lanes x 16 bytes each) per instruction.
        {
            const int ln = fresh(lane);
            const int j = ln & 31, g = ln >> 5, rsub = ln >> 4, piece = ln & 15;
            const float inv = 1.0f / cross_half_sum(l);
            const unsigned region = lds0 + wave * EPI_WAVE;
            const unsigned wr = pin(region + j * EPI_STRIDE + 16 * g);
            const unsigned rd = pin(region + rsub * EPI_STRIDE + 16 * piece);
            const rsrc_t omat = make_rsrc(ohead, (uint32_t)S * (D * 4));      // rows >= S (partial last tile) are dropped
            const unsigned obase = (unsigned)(qrow + rsub) * (D * 4) + 16 * piece;
#pragma unroll
            for (int slab = 0; slab < D / EPI_COLS; ++slab) {
#pragma unroll
                for (int dd = 0; dd < EPI_COLS / 32; ++dd) {
                    const int db = slab * (EPI_COLS / 32) + dd;
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        const v4f val = {o[db][4 * r4] * inv, o[db][4 * r4 + 1] * inv, o[db][4 * r4 + 2] * inv, o[db][4 * r4 + 3] * inv};
                        lds_write<v4f>(wr + 128 * dd + 32 * r4, val);
                    }
                }
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const v4f val = lds_read<v4f>(rd + 4 * i * EPI_STRIDE);
                    buffer_store16(omat, obase + 4 * i * (D * 4) + slab * (EPI_COLS * 4), val);
                }
            }
        }
        __syncthreads();                  // the next item's staging overwrites the epilogue regions
    }
}

// ---------------------------------------------------------------------------------------------
// Host side: pick the instance
// ---------------------------------------------------------------------------------------------
// Number of compute units of the current device (cached per device).
inline int compute_units()
{
    static std::atomic<int> cached[64];               // zero-initialised; every writer stores the same value
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return -1;
    int n = cached[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return -1;
        cached[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

template <int D, int BT, int TPW, int LO, int HI, bool GENERAL, bool PT, bool PVMX = false>
static int launch_variant(const AttnArgs& a, hipStream_t stream)
{
    using C = Cfg<D, BT, TPW>;
    const int N = (a.S + BT - 1) / BT;
    const int64_t items = (int64_t)a.B * a.Hq * ((N + TPW - 1) / TPW);
    if ((!GENERAL && N % TPW != 0) || items <= 0 || items > 0x7fffffffLL) return DMA_ERR_UNSUPPORTED_;
    const int cus = compute_units();
    if (cus <= 0) return DMA_ERR_HIP_;
    // as many workgroups as the chip holds at once (one per CU for the D = 128 instances), each walking its share
    // of the work items
    // per instance, the same on every device of one kind; kept once a query has succeeded (a failed query is repeated by
    // the next call); every writer stores the same value, so several host threads may launch at once
    static std::atomic<int> resident_cache{0};
    int resident = resident_cache.load(std::memory_order_relaxed);
    if (resident == 0) {
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&resident, dma_attn_fwd_kernel<D, BT, TPW, LO, HI, GENERAL, PT, PVMX>, C::T, 0) != hipSuccess || resident <= 0)
            return DMA_ERR_HIP_;
        resident_cache.store(resident, std::memory_order_relaxed);
    }
    const int64_t slots = (int64_t)cus * resident;
    const int64_t blocks = items < slots ? items : slots;
    const float c = (float)(1.4426950408889634074 / sqrt((double)D));
    // ranking blocks: the fewest heads that fill an even number of rounds (mirrors the kernel's view of the grid), in whole
    // groups of query heads that share a kv head: the workers of a round then walk the SAME K/V stream with items of nearly
    // equal length (on the 32k GQA workload 17 % fewer bytes fetched than with single heads, 0.6 % less time)
    const int units = a.B * a.Hkv, group = a.Hq / a.Hkv, NG = (N + TPW - 1) / TPW;
    const bool by_xcd = (units % 8 == 0) && (blocks % 8 == 0);
    const int workers = (int)(by_xcd ? blocks / 8 : blocks);
    const int heads_x = by_xcd ? (units / 8) * group : a.B * a.Hq;
    int head_block = heads_x;
    for (int hb = group; hb < heads_x; hb += group)
        if (heads_x % hb == 0 && ((int64_t)hb * NG) % (2 * workers) == 0) { head_block = hb; break; }
    return launch(dma_attn_fwd_kernel<D, BT, TPW, LO, HI, GENERAL, PT, PVMX>, dim3((unsigned)blocks), dim3(C::T), stream,
                  (const uint16_t*)a.q, (const uint16_t*)a.k, (const uint16_t*)a.v, a.out, a.B, a.Hq, a.Hkv,
                  a.S, a.band, a.sink, a.causal, c, head_block, a.q_amax, a.k_amax);
}

// Alg. 1 as printed (causal, no sink window, sequence a whole number of tile groups) runs the straight-line instance, whose
// tile loads are unbounded; the sink window, the non-causal variant, the per-token scale and a partial last tile run
// the general one, whose loads are bounded by buffer resources (unquantized operands have no per-token scale).
template <int D, int BT, int TPW, int LO, int HI>
static int launch_instance(const AttnArgs& a, hipStream_t stream)
{
    if (a.pv_mx) {
        // the MX-format P V is built for the default pair only, without the per-token scale
        if constexpr (LO == FMT_E2M1 && HI == FMT_E4M3_X) {
            if (a.per_token) return DMA_ERR_UNSUPPORTED_;
            if (a.causal && a.sink == 0 && a.S % (BT * TPW) == 0) return launch_variant<D, BT, TPW, LO, HI, false, false, true>(a, stream);
            return launch_variant<D, BT, TPW, LO, HI, true, false, true>(a, stream);
        } else {
            return DMA_ERR_UNSUPPORTED_;
        }
    }
    if constexpr (LO != FMT_BF16) {
        if (a.per_token) return launch_variant<D, BT, TPW, LO, HI, true, true>(a, stream);
    }
    if (a.causal && a.sink == 0 && a.S % (BT * TPW) == 0) return launch_variant<D, BT, TPW, LO, HI, false, false>(a, stream);
    return launch_variant<D, BT, TPW, LO, HI, true, false>(a, stream);
}

}  // namespace dma
