// Fused forward of Diagonal-Tiled Mixed-Precision Attention for gfx950 (paper, Alg. 1 with the
// online softmax of Sec. 3.2; Q/K quantization of Alg. 2 done in-kernel).
//
// One workgroup owns one logical query tile (B_M = BT rows) of one (batch, query head) and walks the
// key tiles jt = 0 .. it in ascending order: Phase 1 = tiles before the diagonal band in the low
// format, Phase 2 = the last `band` tiles in the high format.  Each wave owns QB blocks of 32 query
// rows.  Everything is computed transposed so that a query row lives in one lane column:
//     S^T[key, query] = K . Q^T      block-scaled MFMA 32x32x64 (A = K codes from LDS, B = Q codes in VGPRs)
//     O^T[d,  query] += V^T . P^T    bf16 MFMA 32x32x16 (A = V^T via LDS transpose reads, B = P^T = the
//                                     exponentiated S^T accumulators, already in operand layout)
// so the row maximum / sum need one cross-half exchange and the running state (m, l) is per lane.
//
// Per key tile: all threads stream K and V (bf16, 16 B per lane, coalesced) into registers one tile
// ahead; K is quantized to the tile's format (block maximum over a lane quad by DPP, E8M0 scale,
// hardware scaled converts) and written to LDS as codes + scale bytes; V goes to LDS as bf16.
#include "dma_device.hpp"
#include "dma_internal.hpp"

namespace dma {

template <int D_, int BT_, int NW_, int QB_>
struct Cfg {
    static constexpr int D = D_, BT = BT_, NW = NW_, QB = QB_;
    static constexpr int T = NW * 64;            // threads per workgroup
    static constexpr int NKB = BT / 32;          // 32-key blocks per key tile
    static constexpr int NDB = D / 32;           // 32-wide blocks of the head dimension (output)
    static constexpr int NH = D / 64;            // k=64 scaled MFMAs per score block
    static constexpr int NKK = D / 16;           // k=16 bf16 MFMAs per score block (BF16 format)
    static constexpr int CPR = D / 8;            // 16-byte chunks per row
    static constexpr int CH = BT * CPR;          // chunks per tile
    static constexpr int CPT = CH / T;           // chunks per thread
    static_assert(NW * QB * 32 == BT, "a workgroup covers exactly one logical query tile");
    static_assert(CH % T == 0, "tile must split evenly over the threads");
    static_assert(D % 64 == 0, "head dimension must be a multiple of 64");
    // LDS row strides in bytes; the padding spreads consecutive rows over the banks.
    static constexpr int KS4 = D / 2 + 16;       // E2M1 codes
    static constexpr int KS8 = D + 16;           // E4M3 codes
    static constexpr int KSB = 2 * D + 16;       // bf16 keys
    static constexpr int VS = 2 * D + 64;        // bf16 values (transpose reads)
    template <int FMT>
    static constexpr int kstride() { return FMT == FMT_E2M1 ? KS4 : FMT == FMT_E4M3 ? KS8 : KSB; }   // bf16 MFMA paths: KSB
};

template <int A, int B>
constexpr int cmax() { return A > B ? A : B; }

// ---------------------------------------------------------------------------------------------
// Query operands of one phase: codes (or bf16) of the wave's QB * 32 rows in MFMA B-operand layout.
// ---------------------------------------------------------------------------------------------
template <typename C, int FMT>
struct QOperand {
    // scaled MFMA: [qb][h] 8 dwords (E2M1 uses the first 4); bf16 MFMA: [qb][kk] 4 dwords.
    static constexpr bool BF = uses_bf16_mfma(FMT);
    v8i mx[BF ? 1 : C::QB][BF ? 1 : C::NH];
    v4i bf[BF ? C::QB : 1][BF ? C::NKK : 1];
    int scale[C::QB];    // byte h = E8M0 of block 2h + g of the lane's row
};

template <typename C, int FMT>
DMA_DEV void load_q(QOperand<C, FMT>& qo, const uint16_t* __restrict__ qhead, int row0, int j, int g, float c)
{
#pragma unroll
    for (int qb = 0; qb < C::QB; ++qb) {
        const uint16_t* rowp = qhead + (int64_t)(row0 + qb * 32 + j) * C::D;
        if constexpr (FMT == FMT_BF16) {
#pragma unroll
            for (int kk = 0; kk < C::NKK; ++kk) qo.bf[qb][kk] = *(const v4i*)(rowp + 16 * kk + 8 * g);
            qo.scale[qb] = 0;
        } else if constexpr (FMT == FMT_E4M3_X) {
            // The lane holds elements 16kk + 8g + [0, 8): MX block b = kk / 2 is spread over both half-waves.
            float x[C::NKK][8];
#pragma unroll
            for (int kk = 0; kk < C::NKK; ++kk) unpack8<true>(*(const v4i*)(rowp + 16 * kk + 8 * g), c, x[kk]);
#pragma unroll
            for (int b = 0; b < C::NKK / 2; ++b) {
                const float amax = cross_half_max(fmaxf(amax8(x[2 * b]), amax8(x[2 * b + 1])));
                const int code = e8m0_code<FMT_E4M3>(amax);
                qo.bf[qb][2 * b] = quant_dequant8_e4m3(x[2 * b], code);
                qo.bf[qb][2 * b + 1] = quant_dequant8_e4m3(x[2 * b + 1], code);
            }
            qo.scale[qb] = 0;
        } else {
            int sc = 0;
            static_for<C::NH>([&](auto H) {
                constexpr int h = H;
                const v4i* src = (const v4i*)(rowp + 32 * (2 * h + g));     // the lane's MX block
                float x[4][8];
                float amax = 0.f;
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    unpack8<true>(src[t], c, x[t]);
                    amax = fmaxf(amax, amax8(x[t]));
                }
                const int code = e8m0_code<FMT>(amax);
                sc |= code << (8 * h);
                v8i r = {0, 0, 0, 0, 0, 0, 0, 0};
                if constexpr (FMT == FMT_E2M1) {
#pragma unroll
                    for (int t = 0; t < 4; ++t) r[t] = encode8_e2m1(x[t], code);
                } else {
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        v2i e = encode8_e4m3(x[t], code);
                        r[2 * t] = e[0];
                        r[2 * t + 1] = e[1];
                    }
                    // E4M3 operand layout: VGPR 0-3 = first half of block 2h (lower lanes) / second half of
                    // block 2h (upper lanes); VGPR 4-7 the same for block 2h+1.  Each lane encoded one whole
                    // block, so the lower lanes' VGPR 4-7 trade places with the upper lanes' VGPR 0-3.
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        int lo = r[t], hi = r[4 + t];
                        swap_halves(lo, hi);
                        r[t] = lo;
                        r[4 + t] = hi;
                    }
                }
                qo.mx[qb][h] = r;
            });
            qo.scale[qb] = sc;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Staging of one key/value tile
// ---------------------------------------------------------------------------------------------
template <typename C>
DMA_DEV void load_tile(v4i (&reg)[C::CPT], const uint16_t* __restrict__ base, int tid)
{
#pragma unroll
    for (int r = 0; r < C::CPT; ++r) {
        const int ch = r * C::T + tid;
        reg[r] = *(const v4i*)(base + (int64_t)ch * 8);          // rows are dense: chunk ch starts at ch * 8
    }
}

template <typename C, int FMT>
DMA_DEV void stage_k(const v4i (&reg)[C::CPT], uint8_t* ldsK, uint8_t* ldsKs, int tid)
{
#pragma unroll
    for (int r = 0; r < C::CPT; ++r) {
        const int ch = r * C::T + tid;
        const int key = ch / C::CPR, dc = ch % C::CPR;
        if constexpr (FMT == FMT_BF16) {
            *(v4i*)(ldsK + key * C::KSB + dc * 16) = reg[r];
        } else {
            float x[8];
            unpack8<false>(reg[r], 1.f, x);
            const float amax = quad_max(amax8(x));
            const int code = e8m0_code<FMT>(amax);
            if constexpr (FMT == FMT_E4M3_X) {
                *(v4i*)(ldsK + key * C::KSB + dc * 16) = quant_dequant8_e4m3(x, code);
                continue;
            }
            if constexpr (FMT == FMT_E2M1) *(int*)(ldsK + key * C::KS4 + dc * 4) = encode8_e2m1(x, code);
            if constexpr (FMT == FMT_E4M3) *(v2i*)(ldsK + key * C::KS8 + dc * 8) = encode8_e4m3(x, code);
            if ((dc & 3) == 0) {
                const int b = dc >> 2;                              // MX block index along D
                ldsKs[key * 8 + 4 * (b & 1) + (b >> 1)] = (uint8_t)code;
            }
        }
    }
}

template <typename C>
DMA_DEV void stage_v(const v4i (&reg)[C::CPT], uint8_t* ldsV, int tid)
{
#pragma unroll
    for (int r = 0; r < C::CPT; ++r) {
        const int ch = r * C::T + tid;
        const int key = ch / C::CPR, dc = ch % C::CPR;
        *(v4i*)(ldsV + key * C::VS + dc * 16) = reg[r];
    }
}

// ---------------------------------------------------------------------------------------------
// One key tile: scores, mask, online softmax, P V
// ---------------------------------------------------------------------------------------------
template <int FMT, int H>
DMA_DEV v16f mfma_mx(const v8i& a, const v8i& b, const v16f& c, int sa, int sb)
{
    constexpr int code = (FMT == FMT_E2M1) ? 4 : 0;
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, code, code, H, sa, H, sb);
}

template <typename C, int FMT>
DMA_DEV void compute_tile(const QOperand<C, FMT>& qo, const uint8_t* ldsK, const uint8_t* ldsKs,
                          const uint8_t* ldsV, bool diagonal, int wave, int lane, float c,
                          float (&m)[C::QB], float (&l)[C::QB], v16f (&o)[C::QB][C::NDB])
{
    const int j = lane & 31, g = lane >> 5;
    v16f s[C::QB][C::NKB];

    // ---- S^T = K . Q^T
#pragma unroll
    for (int kb = 0; kb < C::NKB; ++kb) {
#pragma unroll
        for (int qb = 0; qb < C::QB; ++qb) s[qb][kb] = v16f{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        const int key = kb * 32 + j;
        if constexpr (uses_bf16_mfma(FMT)) {
#pragma unroll
            for (int kk = 0; kk < C::NKK; ++kk) {
                const v4i a = *(const v4i*)(ldsK + key * C::KSB + 32 * kk + 16 * g);
#pragma unroll
                for (int qb = 0; qb < C::QB; ++qb)
                    s[qb][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a),
                                                                        __builtin_bit_cast(v8bf, qo.bf[qb][kk]),
                                                                        s[qb][kb], 0, 0, 0);
            }
            if constexpr (FMT == FMT_BF16) {       // unquantized operands: the softmax factor multiplies the score
#pragma unroll
                for (int qb = 0; qb < C::QB; ++qb) s[qb][kb] *= c;
            }
        } else {
            const int ksc = *(const int*)(ldsKs + key * 8 + 4 * g);
            static_for<C::NH>([&](auto H) {
                constexpr int h = H;
                v8i a = {0, 0, 0, 0, 0, 0, 0, 0};
                if constexpr (FMT == FMT_E2M1) {
                    const v4i lo = *(const v4i*)(ldsK + key * C::KS4 + 16 * (2 * h + g));
                    a[0] = lo[0]; a[1] = lo[1]; a[2] = lo[2]; a[3] = lo[3];
                } else {
                    const v4i lo = *(const v4i*)(ldsK + key * C::KS8 + 64 * h + 16 * g);
                    const v4i hi = *(const v4i*)(ldsK + key * C::KS8 + 64 * h + 32 + 16 * g);
                    a[0] = lo[0]; a[1] = lo[1]; a[2] = lo[2]; a[3] = lo[3];
                    a[4] = hi[0]; a[5] = hi[1]; a[6] = hi[2]; a[7] = hi[3];
                }
#pragma unroll
                for (int qb = 0; qb < C::QB; ++qb)
                    s[qb][kb] = mfma_mx<FMT, h>(a, qo.mx[qb][h], s[qb][kb], ksc, qo.scale[qb]);
            });
        }
    }

    // ---- causal mask on the tile that straddles the diagonal: key > query -> -inf
    if (diagonal) {
#pragma unroll
        for (int qb = 0; qb < C::QB; ++qb) {
            const int qi = (wave * C::QB + qb) * 32 + j;
#pragma unroll
            for (int kb = 0; kb < C::NKB; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int kj = kb * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
                    if (kj > qi) s[qb][kb][r] = -INFINITY;
                }
        }
    }

    // ---- online softmax in base 2
#pragma unroll
    for (int qb = 0; qb < C::QB; ++qb) {
        float mx = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < C::NKB; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[qb][kb][r]);
        mx = cross_half_max(mx);
        const float mnew = fmaxf(m[qb], mx);
        const float alpha = __builtin_amdgcn_exp2f(m[qb] - mnew);
        m[qb] = mnew;
        float psum = 0.f;
#pragma unroll
        for (int kb = 0; kb < C::NKB; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float p = __builtin_amdgcn_exp2f(s[qb][kb][r] - mnew);
                psum += p;
                s[qb][kb][r] = p;
            }
        l[qb] = l[qb] * alpha + psum;
#pragma unroll
        for (int db = 0; db < C::NDB; ++db) o[qb][db] *= alpha;
    }

    // ---- O^T += V^T . P^T
    const int l16 = lane & 15, q16 = lane >> 4;
    // transpose read: lane l16 of a 16-lane group points at row (l16 / 4) of a 4-key x 16-column patch
    const uint8_t* vlane = ldsV + (4 * g + (l16 >> 2)) * C::VS + 2 * (16 * (q16 & 1) + 4 * (l16 & 3));
#pragma unroll
    for (int kb = 0; kb < C::NKB; ++kb) {
#pragma unroll
        for (int cc = 0; cc < 2; ++cc) {
            v8bf pb[C::QB];
#pragma unroll
            for (int qb = 0; qb < C::QB; ++qb) {
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    v2f f = {s[qb][kb][8 * cc + 2 * t], s[qb][kb][8 * cc + 2 * t + 1]};
                    v2bf h2 = __builtin_convertvector(f, v2bf);
                    pb[qb][2 * t] = h2[0];
                    pb[qb][2 * t + 1] = h2[1];
                }
            }
            const uint8_t* vk = vlane + (kb * 32 + cc * 16) * C::VS;
#pragma unroll
            for (int db = 0; db < C::NDB; ++db) {
                typedef __attribute__((address_space(3))) v4s lds_v4s;
                const v4s a0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s*)(vk + 64 * db));
                const v4s a1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s*)(vk + 8 * C::VS + 64 * db));
                v8s a;
                a[0] = a0[0]; a[1] = a0[1]; a[2] = a0[2]; a[3] = a0[3];
                a[4] = a1[0]; a[5] = a1[1]; a[6] = a1[2]; a[7] = a1[3];
#pragma unroll
                for (int qb = 0; qb < C::QB; ++qb)
                    o[qb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a), pb[qb],
                                                                        o[qb][db], 0, 0, 0);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// One phase of Alg. 1: key tiles [jt0, jt1) in format FMT
// ---------------------------------------------------------------------------------------------
template <typename C, int FMT>
DMA_DEV void run_phase(const uint16_t* __restrict__ qhead, const uint16_t* __restrict__ khead,
                       const uint16_t* __restrict__ vhead, int it, int jt0, int jt1, float c,
                       uint8_t* ldsK, uint8_t* ldsKs, uint8_t* ldsV, int tid, int wave, int lane,
                       float (&m)[C::QB], float (&l)[C::QB], v16f (&o)[C::QB][C::NDB])
{
    if (jt0 >= jt1) return;
    QOperand<C, FMT> qo;
    load_q<C, FMT>(qo, qhead, it * C::BT + wave * C::QB * 32, lane & 31, lane >> 5, c);

    v4i kreg[C::CPT], vreg[C::CPT];
    load_tile<C>(kreg, khead + (int64_t)jt0 * C::BT * C::D, tid);
    load_tile<C>(vreg, vhead + (int64_t)jt0 * C::BT * C::D, tid);
    for (int jt = jt0; jt < jt1; ++jt) {
        stage_k<C, FMT>(kreg, ldsK, ldsKs, tid);
        stage_v<C>(vreg, ldsV, tid);
        __syncthreads();
        if (jt + 1 < jt1) {                       // next tile's global loads fly during the compute
            load_tile<C>(kreg, khead + (int64_t)(jt + 1) * C::BT * C::D, tid);
            load_tile<C>(vreg, vhead + (int64_t)(jt + 1) * C::BT * C::D, tid);
        }
        compute_tile<C, FMT>(qo, ldsK, ldsKs, ldsV, jt == it, wave, lane, c, m, l, o);
        __syncthreads();
    }
}

template <int D, int BT, int NW, int QB, int LO, int HI>
__global__ void __launch_bounds__(NW * 64)
dma_attn_fwd_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                    const uint16_t* __restrict__ v, float* __restrict__ out,
                    int B, int Hq, int Hkv, int S, int band, float c)
{
    using C = Cfg<D, BT, NW, QB>;
    constexpr int KBYTES = BT * cmax<C::template kstride<LO>(), C::template kstride<HI>()>();
    __shared__ __attribute__((aligned(16))) uint8_t ldsK[KBYTES];
    __shared__ __attribute__((aligned(16))) uint8_t ldsKs[BT * 8];
    __shared__ __attribute__((aligned(16))) uint8_t ldsV[BT * C::VS];

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;

    // ---- which (batch, query head, query tile): heaviest tiles first; when the (batch, kv head) units
    // divide over the 8 XCDs, every unit stays on one XCD so its K/V stream is shared in that L2.
    const int N = S / BT;
    const int group = Hq / Hkv;
    const int units = B * Hkv;
    const int bid = blockIdx.x;
    int b, hq, it;
    if (units % 8 == 0) {
        const int xcd = bid & 7, idx = bid >> 3;
        const int per_unit = group * N;
        const int unit = (idx / per_unit) * 8 + xcd, rem = idx % per_unit;
        b = unit / Hkv;
        hq = (unit % Hkv) * group + rem / N;
        it = N - 1 - rem % N;
    } else {
        const int bh = bid % (B * Hq);
        it = N - 1 - bid / (B * Hq);
        b = bh / Hq;
        hq = bh % Hq;
    }
    const int hkv = hq / group;
    const uint16_t* qhead = q + ((int64_t)b * Hq + hq) * S * D;
    const uint16_t* khead = k + ((int64_t)b * Hkv + hkv) * S * D;
    const uint16_t* vhead = v + ((int64_t)b * Hkv + hkv) * S * D;
    float* ohead = out + ((int64_t)b * Hq + hq) * S * D;

    float m[QB], l[QB];
    v16f o[QB][C::NDB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        m[qb] = -INFINITY;
        l[qb] = 0.f;          // Alg. 1 starts l at 1; the first rescale factor 2^(-inf) erases it
#pragma unroll
        for (int db = 0; db < C::NDB; ++db) o[qb][db] = v16f{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    }

    // ---- Phase 1 (low format) then Phase 2 (high format, the last `band` key tiles)
    const int lo_end = max(0, it + 1 - band);
    if constexpr (LO == HI) {
        run_phase<C, LO>(qhead, khead, vhead, it, 0, it + 1, c, ldsK, ldsKs, ldsV, tid, wave, lane, m, l, o);
    } else {
        run_phase<C, LO>(qhead, khead, vhead, it, 0, lo_end, c, ldsK, ldsKs, ldsV, tid, wave, lane, m, l, o);
        run_phase<C, HI>(qhead, khead, vhead, it, lo_end, it + 1, c, ldsK, ldsKs, ldsV, tid, wave, lane, m, l, o);
    }

    // ---- O / l
    const int j = lane & 31, g = lane >> 5;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const float inv = 1.0f / cross_half_sum(l[qb]);
        float* orow = ohead + (int64_t)(it * BT + (wave * QB + qb) * 32 + j) * D;
#pragma unroll
        for (int db = 0; db < C::NDB; ++db)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                v4f val = {o[qb][db][4 * r4] * inv, o[qb][db][4 * r4 + 1] * inv, o[qb][db][4 * r4 + 2] * inv,
                           o[qb][db][4 * r4 + 3] * inv};
                *(v4f*)(orow + 32 * db + 8 * r4 + 4 * g) = val;
            }
    }
}

// ---------------------------------------------------------------------------------------------
// Host side: pick the instance
// ---------------------------------------------------------------------------------------------
template <int D, int BT, int NW, int QB, int LO, int HI>
static int launch_instance(const AttnArgs& a, hipStream_t stream)
{
    const int N = a.S / BT;
    const int64_t blocks = (int64_t)a.B * a.Hq * N;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return DMA_ERR_UNSUPPORTED_;
    const float c = (float)(1.4426950408889634074 / sqrt((double)D));
    hipLaunchKernelGGL((dma_attn_fwd_kernel<D, BT, NW, QB, LO, HI>), dim3((unsigned)blocks), dim3(NW * 64), 0, stream,
                       (const uint16_t*)a.q, (const uint16_t*)a.k, (const uint16_t*)a.v, a.out, a.B, a.Hq, a.Hkv,
                       a.S, a.band, c);
    return hipGetLastError() == hipSuccess ? DMA_OK_ : DMA_ERR_HIP_;
}

template <int D, int BT, int NW, int QB>
static int launch_formats(const AttnArgs& a, hipStream_t stream)
{
    const int lo = a.lo_fmt, hi = a.hi_fmt;
    // a.lo_fmt / a.hi_fmt arrive as internal product-path ids (FMT_*).
    if (lo == FMT_E2M1 && hi == FMT_E4M3_X) return launch_instance<D, BT, NW, QB, FMT_E2M1, FMT_E4M3_X>(a, stream);
    if (lo == FMT_E2M1 && hi == FMT_E4M3) return launch_instance<D, BT, NW, QB, FMT_E2M1, FMT_E4M3>(a, stream);
    if (lo == FMT_E2M1 && hi == FMT_E2M1) return launch_instance<D, BT, NW, QB, FMT_E2M1, FMT_E2M1>(a, stream);
    if (lo == FMT_E4M3_X && hi == FMT_E4M3_X) return launch_instance<D, BT, NW, QB, FMT_E4M3_X, FMT_E4M3_X>(a, stream);
    if (lo == FMT_E4M3 && hi == FMT_E4M3) return launch_instance<D, BT, NW, QB, FMT_E4M3, FMT_E4M3>(a, stream);
    if (lo == FMT_BF16 && hi == FMT_BF16) return launch_instance<D, BT, NW, QB, FMT_BF16, FMT_BF16>(a, stream);
    return DMA_ERR_UNSUPPORTED_;
}

int launch_attn_fwd(const AttnArgs& a, hipStream_t stream)
{
    if (a.D == 128 && a.tile == 128) return launch_formats<128, 128, 4, 1>(a, stream);
    if (a.D == 64 && a.tile == 64) return launch_formats<64, 64, 2, 1>(a, stream);
    return DMA_ERR_UNSUPPORTED_;
}

}  // namespace dma
