// bf16 MFMA implicit-GEMM convolution for gfx950 (CDNA4): forward / dgrad ("gather" form) and
// wgrad.  fp32 accumulation in v_mfma_f32_32x32x16_bf16; operands staged through LDS.
//
// Gather form (forward and dgrad share it, see GatherConv):
//     out[pixel][ko] = sum_k  X[pixel][k] * Wt[ko][k],   k = (r, s, ki), ki fastest
// is a GEMM whose K index is contiguous in memory for both operands (NHWC activations,
// [Ko][R][S][Ki] filters), which is exactly the per-lane fragment the MFMA wants (8 consecutive
// k for one row).  A block owns BP output pixels x BC output channels; 16-byte chunks of the
// operand rows travel from HBM/L2 straight into LDS (buffer_load ... lds, no register staging)
// into a ring of three K-tiles; the XOR swizzle that makes the ds_read_b128 fragment loads
// bank-conflict free is applied on the global side, by choosing which chunk a lane fetches.
// The MFMA's A operand is the filter tile and its B operand the pixel tile, so a lane ends up
// with 4 consecutive output channels of one pixel per accumulator quad; the tile is then
// staged through LDS as [pixel][channel] to leave the kernel as 16-byte, fully coalesced rows
// (with bias / ReLU, or with the gradient epilogue: accumulate + ReLU gate of the producer).
//
// wgrad:  dw[ko][r][s][c] += sum_pixels dy[pixel][ko] * x[pixel @ tap (r,s)][c]
// contracts over pixels, which are NOT contiguous for either operand: tiles are stored in LDS
// as [pixel][channel] exactly as they come from HBM, and the fragments are fetched with the
// CDNA4 transposing LDS read (ds_read_b64_tr_b16), which hands each lane 4 consecutive
// pixels of one channel.  The pixel range is split over blocks (split-K); partial sums go to
// a workspace and a second kernel adds them in a fixed order into the fp32 accumulators.
#include "kernels.h"
#include "mfma_common.h"

namespace bapipe {
namespace {

template <int BK> __device__ __forceinline__ int swz(int row)
{
    // 16-byte slots of 16 consecutive rows must fall into 16 different bank groups
    return BK == 32 ? ((row >> 2) & 3) : ((row >> 1) & 7);
}

// ------------------------------------------------------------------------------------------
// gather convolution
// ------------------------------------------------------------------------------------------
// The operand tiles travel HBM/L2 -> LDS without touching registers: buffer_load_dwordx4 ... lds
// writes the 64 lanes' 16-byte chunks to 64 consecutive LDS slots starting at a wave-uniform
// address, and a lane whose offset is outside the buffer gets zeros (that is the zero padding of
// the convolution and the ragged tile edges).  The XOR swizzle of the tile layout is applied by
// choosing WHICH chunk a lane fetches, since WHERE it lands is fixed by the lane id.
// STAGES tiles form a ring; tile kt+STAGES-1 is requested right after the barrier that retires
// tile kt-1, so STAGES-1 K-tiles of latency are covered while the MFMAs run.
template <int BP, int BC, int WP, int WC, int BK, int STAGES, bool S1, bool TAPS_INNER>
__global__ __launch_bounds__(WP *WC * 64, WP *WC >= 8 ? 1 : 2) void k_gather_mfma(
    const bf16_t *__restrict__ in, const bf16_t *__restrict__ wt, const float *__restrict__ bias,
    bf16_t *out, const bf16_t *__restrict__ gate, int accum, int relu, int is_grad, GatherConv g,
    int tiles_c, unsigned in_bytes, unsigned wt_bytes, float *__restrict__ part, int kt_per_split,
    float *__restrict__ stat_part, const bf16_t *__restrict__ bn_x, const float *__restrict__ bn_stats,
    const bf16_t *old_from)
{
    constexpr int NT = WP * WC * 64, NW = WP * WC;
    constexpr int CPR = BK / 8;              // 16-byte chunks per tile row
    constexpr int RPW = 64 / CPR;            // tile rows one wave-wide load covers
    constexpr int XL = BP / (RPW * NW);      // loads per wave for the pixel tile
    constexpr int WL = BC / (RPW * NW);      // loads per wave for the filter tile
    constexpr int WT_P = BP / WP, WT_C = BC / WC;
    constexpr int TP = WT_P / 32, TC = WT_C / 32;
    constexpr int KSUB = BK / 16;
    constexpr int SROW = BC + 4;             // staging row (elements): 8-byte aligned, odd multiple of 8 bytes
    constexpr int STAGE_ELEMS = (BP + BC) * BK;
    static_assert(XL >= 1 && WL >= 1 && BP % (RPW * NW) == 0 && BC % (RPW * NW) == 0, "tile/thread mismatch");
    static_assert(BK == 32, "swizzle below assumes 4 chunks per row");

    extern __shared__ __align__(16) unsigned char smem[];
    const lds_addr_of lds_of(smem);
    uint16_t *ring = reinterpret_cast<uint16_t *>(smem);               // [STAGES][ W tile | X tile ]
    uint16_t *sO = reinterpret_cast<uint16_t *>(smem);                 // [BP][SROW] (epilogue, reuses the ring)
    constexpr size_t RING_BYTES = (size_t)STAGES * STAGE_ELEMS * 2, EPI_BYTES = (size_t)BP * SROW * 2;
    float *sBias = reinterpret_cast<float *>(smem + (RING_BYTES > EPI_BYTES ? RING_BYTES : EPI_BYTES));   // [BC]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wp = wave % WP, wc = wave / WP;
    // slot (row, c') a lane fills inside one wave-wide load, and the chunk column it must fetch
    const int lrow = lane >> 2;
    const int lc = (lane & 3) ^ ((lane >> 4) & 3);       // = c' ^ swz(row); the same for every load

    // split-K: blockIdx.y owns K-tiles [kt0, kt1) and leaves fp32 partial sums in part[split][pixel][co]
    const int bid = xcd_remap(blockIdx.x, gridDim.x);
    const int tile_c = bid % tiles_c, tile_p = bid / tiles_c;
    const int co0 = tile_c * BC;
    const int pix0 = tile_p * BP;                    // pixel counts fit 31 bits (checked by the launcher)
    const int npix = g.N * g.Ho * g.Wo;
    const int K = g.R * g.S * g.Ci;
    const int KT = TAPS_INNER ? (g.Ci / BK) * g.R * g.S : (K + BK - 1) / BK;
    constexpr unsigned OOB = 0x80000000u;

    __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(in), 0, (int)in_bytes, 0x00020000);
    __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(wt), 0, (int)wt_bytes, 0x00020000);

    // ---- per-lane gather state: the pixel rows this lane fetches (row = (i*NW + wave)*RPW + lrow)
    // FAST (stride 1, taps innermost, at most 32 taps): everything that depends on the lane is
    // computed once - the byte offset of the lane's chunk at tap (0,0) and a bit mask of the taps
    // that fall inside the image - so that a K-tile costs one scalar offset, one mask test and one
    // add per load.
    constexpr bool FAST = S1 && TAPS_INNER;
    int hb[XL], wb[XL];
    unsigned xoff[XL];                       // generic: byte offset of pixel (n, 0, 0), channel 0; FAST: see above
    unsigned tapmask[XL];
#pragma unroll
    for (int i = 0; i < XL; ++i) {
        int p = pix0 + (i * NW + wave) * RPW + lrow;
        tapmask[i] = 0;
        if (p < npix) {
            int ow = p % g.Wo;
            int t = p / g.Wo;
            int oh = t % g.Ho;
            int n = t / g.Ho;
            hb[i] = oh * g.s_out - g.pad_h;
            wb[i] = ow * g.s_out - g.pad_w;
            xoff[i] = (unsigned)n * (unsigned)(g.Hi * g.Wi * g.Ci) * 2u;
            if (FAST) {
                for (int r = 0; r < g.R; ++r)
                    for (int q = 0; q < g.S; ++q)
                        if ((unsigned)(hb[i] + r) < (unsigned)g.Hi && (unsigned)(wb[i] + q) < (unsigned)g.Wi)
                            tapmask[i] |= 1u << (r * g.S + q);
                xoff[i] += (unsigned)((hb[i] * g.Wi + wb[i]) * g.Ci + 8 * lc) * 2u;     // may wrap; the tap offset undoes it
            }
        } else {
            hb[i] = -(1 << 28);          // fails every bounds check below
            wb[i] = 0;
            xoff[i] = 0;
        }
    }
    unsigned woff[WL];
#pragma unroll
    for (int i = 0; i < WL; ++i) {
        int co = co0 + (i * NW + wave) * RPW + lrow;
        woff[i] = co < g.Co ? (unsigned)co * (unsigned)K * 2u : OOB;
        if (FAST && co < g.Co) woff[i] += 16u * lc;
    }
    // K order.  TAPS_INNER (Ci a multiple of BK): tile kt covers channels [cit*BK, +BK) of tap
    // (kt % RS), taps innermost, so that consecutive tiles re-read almost the same pixels (shifted
    // by one column / one row) and hit in the CU's vector L1.  Otherwise k = (r, s, ci) flattened,
    // ci fastest, and a tile may straddle taps.  Both operands use the same order.
    const int kt0 = part ? blockIdx.y * kt_per_split : 0;
    const int kt1 = part ? (kt0 + kt_per_split < KT ? kt0 + kt_per_split : KT) : KT;
    int kk = kt0 * BK + 8 * lc;                        // flattened k of this lane's chunk (generic order)
    int kr = kk / (g.S * g.Ci), ks = (kk / g.Ci) % g.S, kc = kk % g.Ci;
    int cb = 0;                                        // FAST: first channel of the tile (wave-uniform)
    if (TAPS_INNER) {
        const int tap = kt0 % (g.R * g.S);
        kr = tap / g.S;
        ks = tap % g.S;
        cb = (kt0 / (g.R * g.S)) * BK;
        kc = cb + 8 * lc;                              // channel offset; tap = (kr, ks)
    }

    auto issue_tile = [&](int stage) {
        uint16_t *sw = ring + stage * STAGE_ELEMS, *sx = sw + BC * BK;
        if constexpr (FAST) {
            const bool kin = cb < g.Ci;
            const int tap = kr * g.S + ks;
            const unsigned bit = kin ? 1u << tap : 0u;
            const unsigned xo = (unsigned)((kr * g.Wi + ks) * g.Ci + cb) * 2u;
            const unsigned wo = kin ? (unsigned)(tap * g.Ci + cb) * 2u : OOB;
#pragma unroll
            for (int i = 0; i < XL; ++i) {
                unsigned vo = (tapmask[i] & bit) ? xoff[i] + xo : OOB;
                dma16(xrsrc, lds_of(sx + (i * NW + wave) * RPW * BK), vo);
            }
#pragma unroll
            for (int i = 0; i < WL; ++i) {
                unsigned vo = (woff[i] + wo) | (woff[i] & OOB);       // rows past Co stay out of range
                if (!kin) vo = OOB;                                   // and so do tiles past K
                dma16(wrsrc, lds_of(sw + (i * NW + wave) * RPW * BK), vo);
            }
            return;                                   // the caller advances (kr, ks, cb) after its MFMAs
        }
        const bool kin = TAPS_INNER ? (kc < g.Ci) : (kr < g.R);
        const unsigned koff = (unsigned)(TAPS_INNER ? (kr * g.S + ks) * g.Ci + kc : kk) * 2u;
#pragma unroll
        for (int i = 0; i < XL; ++i) {
            int hn = hb[i] + kr, wn = wb[i] + ks;
            int ih, iw;
            bool ok;
            if (S1) {
                ih = hn;
                iw = wn;
                ok = kin && (unsigned)ih < (unsigned)g.Hi && (unsigned)iw < (unsigned)g.Wi;
            } else {
                ih = hn / g.s_in;
                iw = wn / g.s_in;
                ok = kin && hn >= 0 && wn >= 0 && ih * g.s_in == hn && iw * g.s_in == wn && ih < g.Hi && iw < g.Wi;
            }
            unsigned vo = ok ? xoff[i] + (unsigned)((ih * g.Wi + iw) * g.Ci + kc) * 2u : OOB;
            dma16(xrsrc, lds_of(sx + (i * NW + wave) * RPW * BK), vo);
        }
#pragma unroll
        for (int i = 0; i < WL; ++i) {
            unsigned vo = (kin && woff[i] != OOB) ? woff[i] + koff : OOB;
            dma16(wrsrc, lds_of(sw + (i * NW + wave) * RPW * BK), vo);
        }
        // advance to the next K-tile
        if (TAPS_INNER) {
            if (++ks == g.S) {
                ks = 0;
                if (++kr == g.R) {
                    kr = 0;
                    kc += BK;
                }
            }
        } else {
            kk += BK;
            kc += BK;
            while (kc >= g.Ci) {
                kc -= g.Ci;
                if (++ks == g.S) {
                    ks = 0;
                    ++kr;
                }
            }
        }
    };
    // FAST path: step (kr, ks, cb) to the next K-tile.  Kept apart from issue_tile so that the branchy
    // scalar code does not split the block in which the MFMAs and the address arithmetic interleave.
    auto advance_tile = [&]() {
        if (FAST) {
            if (++ks == g.S) {
                ks = 0;
                if (++kr == g.R) {
                    kr = 0;
                    cb += BK;
                }
            }
        }
    };

    f32x16_t acc[TC][TP];
#pragma unroll
    for (int a = 0; a < TC; ++a)
#pragma unroll
        for (int b = 0; b < TP; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;

    const int frow = lane & 31, fhalf = lane >> 5;
    // operand fragments of K-sub-step ks16 of the tile in ring slot `stage`
    auto load_frags = [&](int stage, int ks16, bf16x8_t(&fa)[TC], bf16x8_t(&fb)[TP]) {
        const uint16_t *cw = ring + stage * STAGE_ELEMS, *cx = cw + BC * BK;
        const int ch = 2 * ks16 + fhalf;
#pragma unroll
        for (int a = 0; a < TC; ++a) {
            int row = wc * WT_C + a * 32 + frow;
            fa[a] = as_frag(*reinterpret_cast<const chunk16 *>(cw + row * BK + ((ch ^ swz<BK>(row)) << 3)));
        }
#pragma unroll
        for (int b = 0; b < TP; ++b) {
            int row = wp * WT_P + b * 32 + frow;
            fb[b] = as_frag(*reinterpret_cast<const chunk16 *>(cx + row * BK + ((ch ^ swz<BK>(row)) << 3)));
        }
    };
    auto mfma_all = [&](const bf16x8_t(&fa)[TC], const bf16x8_t(&fb)[TP]) {
#pragma unroll
        for (int a = 0; a < TC; ++a)
#pragma unroll
            for (int b = 0; b < TP; ++b)
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
    };

    // the block's bias slice goes to LDS now; it is read after the barriers of the main loop
    if (tid < BC) sBias[tid] = (bias && co0 + tid < g.Co) ? bias[co0 + tid] : 0.0f;

    // Software pipeline.  The ring holds STAGES tiles in flight or in use; every iteration requests
    // exactly XL+WL loads per wave (tiles past the end fetch zeros nobody multiplies), so "at most
    // (STAGES-2)*(XL+WL) outstanding" means the next tile has landed.  Fragments are double-buffered
    // in registers: the LDS reads of a sub-step are issued one sub-step (one group of MFMAs) before
    // they are needed, and the barrier that publishes tile kt+1 sits between the two MFMA groups of
    // tile kt.  By then every wave holds all of tile kt in registers, so its slot is refilled at once.
    // sched_barrier pins that order: left alone the scheduler sinks the reads next to their MFMAs.
    static_assert(KSUB == 2, "pipeline below is written for two sub-steps per tile");
    constexpr int NLOAD = XL + WL;
#pragma unroll
    for (int st = 0; st < STAGES; ++st) {
        issue_tile(st);
        advance_tile();
    }
    WAIT_VMCNT((STAGES - 1) * NLOAD);
    WAIT_LGKMCNT(0);       // no scalar load may be pending at loop entry, or every LDS wait in the loop becomes a full drain
    __builtin_amdgcn_s_barrier();
    bf16x8_t fa0[TC], fb0[TP], fa1[TC], fb1[TP];
    load_frags(0, 0, fa0, fb0);
    int rd = 0;
    for (int kt = kt0; kt < kt1; ++kt) {
        const int nx = rd + 1 == STAGES ? 0 : rd + 1;
        load_frags(rd, 1, fa1, fb1);
        __builtin_amdgcn_sched_barrier(0);            // keep the reads ahead of the MFMAs that hide them
        mfma_all(fa0, fb0);
        __builtin_amdgcn_sched_barrier(0);
        WAIT_LGKMCNT(0);                              // this wave has read all of tile kt
        WAIT_VMCNT((STAGES - 2) * NLOAD);             // its share of tile kt+1 has landed
        __builtin_amdgcn_s_barrier();
        load_frags(nx, 0, fa0, fb0);
        __builtin_amdgcn_sched_barrier(0);
        issue_tile(rd);                               // tile kt+STAGES into the slot just retired; its address
        mfma_all(fa1, fb1);                           // arithmetic is free to mix with these MFMAs
        __builtin_amdgcn_sched_barrier(0);
        advance_tile();
        rd = nx;
    }
    WAIT_VMCNT(0);
    __syncthreads();

    if (part) {
        // split-K: raw fp32 sums, 4 consecutive channels of one pixel per store; bias, ReLU and the
        // gradient epilogue are applied by the reduction kernel
        float *dst = part + (size_t)blockIdx.y * npix * g.Co;
#pragma unroll
        for (int a = 0; a < TC; ++a)
#pragma unroll
            for (int b = 0; b < TP; ++b) {
                const int p = pix0 + wp * WT_P + b * 32 + frow;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int co = co0 + wc * WT_C + a * 32 + 8 * q + 4 * fhalf;
                    if (p < npix && co < g.Co)
                        *reinterpret_cast<float4 *>(dst + (size_t)p * g.Co + co) =
                            make_float4(acc[a][b][4 * q], acc[a][b][4 * q + 1], acc[a][b][4 * q + 2], acc[a][b][4 * q + 3]);
                }
            }
        return;
    }

    // ---- epilogue: every wave parks its sub-tile in LDS as [pixel][channel] (bf16, bias and ReLU
    // applied), one barrier, then the block streams the tile out as 16-byte coalesced rows
    const chunk16 zero16 = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int a = 0; a < TC; ++a) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int col = wc * WT_C + a * 32 + 8 * q + 4 * fhalf;      // channel inside the tile
            const float4 bv = *reinterpret_cast<const float4 *>(sBias + col);
#pragma unroll
            for (int b = 0; b < TP; ++b) {
                const int prow = wp * WT_P + b * 32 + frow;              // pixel inside the tile
                float v0 = acc[a][b][4 * q] + bv.x, v1 = acc[a][b][4 * q + 1] + bv.y;
                float v2 = acc[a][b][4 * q + 2] + bv.z, v3 = acc[a][b][4 * q + 3] + bv.w;
                if (relu) {
                    v0 = fmaxf(v0, 0.0f);
                    v1 = fmaxf(v1, 0.0f);
                    v2 = fmaxf(v2, 0.0f);
                    v3 = fmaxf(v3, 0.0f);
                }
                chunk8 c8;
                c8[0] = (uint32_t)f32_to_bf16_bits(v0) | ((uint32_t)f32_to_bf16_bits(v1) << 16);
                c8[1] = (uint32_t)f32_to_bf16_bits(v2) | ((uint32_t)f32_to_bf16_bits(v3) << 16);
                *reinterpret_cast<chunk8 *>(sO + prow * SROW + col) = c8;
            }
        }
    }
    // gradient epilogue: the ReLU-gate rows of the thread's first units are requested now, so that they travel
    // while the staging tile is being completed instead of after the barrier
    constexpr int GUNITS = BP * (BC / 8) / NT, GPRE = GUNITS < 8 ? GUNITS : 8;
    chunk16 gpre[GPRE];
    if (is_grad && gate) {
#pragma unroll
        for (int it = 0; it < GPRE; ++it) {
            const int u = tid + it * NT;
            const int p = pix0 + u / (BC / 8), co = co0 + (u % (BC / 8)) * 8;
            gpre[it] = (p < npix && co < g.Co) ? *reinterpret_cast<const chunk16 *>(gate + (size_t)p * g.Co + co) : zero16;
        }
    }
    __syncthreads();
    // Per-channel sum and sum of squares of the STORED (rounded) values of this pixel tile, for a batch-norm
    // that follows: stat_part[q][pixel tile][channel], q = 0 sum, 1 squares - the layout the final pass of the
    // column reductions reads.  One thread per channel walks down the staged tile.
    if (stat_part && !bn_x) {
        for (int cc = tid; cc < BC; cc += NT) {
            const int co = co0 + cc;
            if (co < g.Co) {
                const int rows = npix - pix0 < BP ? npix - pix0 : BP;
                float s1 = 0.0f, s2 = 0.0f;
                for (int r = 0; r < rows; ++r) {
                    const float v = __uint_as_float((uint32_t)sO[r * SROW + cc] << 16);
                    s1 += v;
                    s2 += v * v;
                }
                const int tiles_p = (int)gridDim.x / tiles_c;
                stat_part[(size_t)tile_p * g.Co + co] = s1;
                stat_part[((size_t)tiles_p + tile_p) * g.Co + co] = s2;
            }
        }
    }
    constexpr int CH8 = BC / 8;                 // 16-byte units per pixel row
    constexpr int UNITS = BP * CH8 / NT;        // per thread
    static_assert(NT % CH8 == 0, "a thread keeps one channel group through the loop below");
    // bn_x: the gradient written here is the output gradient of a batch-norm whose input is bn_x and whose
    // (mean, 1/std) are bn_stats: the per-channel sums of dy and dy*xhat over this pixel tile are taken on
    // the way out (what the first pass of the batch-norm's backward would compute from HBM)
    float bs1[8], bs2[8], bmu[8], binv[8];
    if (bn_x) {
        const int co = co0 + (tid % CH8) * 8;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            bs1[j] = bs2[j] = 0.0f;
            bmu[j] = co + j < g.Co ? bn_stats[co + j] : 0.0f;
            binv[j] = co + j < g.Co ? bn_stats[g.Co + co + j] : 0.0f;
        }
    }
#pragma unroll
    for (int it = 0; it < UNITS; ++it) {
        const int u = tid + it * NT;
        const int prow = u / CH8, c8i = u % CH8;
        const int p = pix0 + prow;
        const int co = co0 + c8i * 8;
        if (p < npix && co < g.Co) {
            chunk8 lo = *reinterpret_cast<const chunk8 *>(sO + prow * SROW + c8i * 8);
            chunk8 hi = *reinterpret_cast<const chunk8 *>(sO + prow * SROW + c8i * 8 + 4);
            chunk16 v = {lo[0], lo[1], hi[0], hi[1]};
            bf16_t *dst = out + (size_t)p * g.Co + co;
            if (is_grad) {
                chunk16 old = zero16, gt = zero16, r;
                if (accum) old = *reinterpret_cast<const chunk16 *>(old_from ? old_from + (size_t)p * g.Co + co : dst);
                if (gate) gt = it < GPRE ? gpre[it < GPRE ? it : 0] : *reinterpret_cast<const chunk16 *>(gate + (size_t)p * g.Co + co);
#pragma unroll
                for (int j = 0; j < 4; ++j) r[j] = grad_epilogue_pair(v[j], old[j], gt[j], accum != 0, gate != nullptr);
                *reinterpret_cast<chunk16 *>(dst) = r;
                if (bn_x) {
                    const chunk16 xv = *reinterpret_cast<const chunk16 *>(bn_x + (size_t)p * g.Co + co);
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const float gj = __uint_as_float((j & 1) ? (r[j >> 1] & 0xFFFF0000u) : (r[j >> 1] << 16));
                        const float xj = __uint_as_float((j & 1) ? (xv[j >> 1] & 0xFFFF0000u) : (xv[j >> 1] << 16));
                        bs1[j] += gj;
                        bs2[j] += gj * ((xj - bmu[j]) * binv[j]);
                    }
                }
            } else {
                *reinterpret_cast<chunk16 *>(dst) = v;
            }
        }
    }
    if (bn_x) {
        // combine the NT / CH8 threads that share a channel group through LDS (the staging tile is free now)
        constexpr int RG = NT / CH8;
        static_assert((size_t)RG * BC * 2 * sizeof(float) <= EPI_BYTES, "reduction buffer fits the staging tile");
        float *red = reinterpret_cast<float *>(smem);                      // [RG][2][BC]
        __syncthreads();
        const int rg = tid / CH8, c8i = tid % CH8;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            red[(rg * 2 + 0) * BC + c8i * 8 + j] = bs1[j];
            red[(rg * 2 + 1) * BC + c8i * 8 + j] = bs2[j];
        }
        __syncthreads();
        for (int cc = tid; cc < BC; cc += NT) {
            const int co = co0 + cc;
            if (co < g.Co) {
                float t1 = 0.0f, t2 = 0.0f;
                for (int k = 0; k < RG; ++k) {
                    t1 += red[(k * 2 + 0) * BC + cc];
                    t2 += red[(k * 2 + 1) * BC + cc];
                }
                const int tiles_p = (int)gridDim.x / tiles_c;
                stat_part[(size_t)tile_p * g.Co + co] = t1;
                stat_part[((size_t)tiles_p + tile_p) * g.Co + co] = t2;
            }
        }
    }
}

// out[p][co] = epilogue( sum_split part[split][p][co] + bias[co] ), 8 channels per thread
__global__ void k_gather_splitk_reduce(const float *__restrict__ part, int splits, size_t total, int Co,
                                       const float *__restrict__ bias, bf16_t *out,
                                       const bf16_t *__restrict__ gate, int accum, int relu, int is_grad,
                                       const bf16_t *old_from)
{
    size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 8;
    if (i >= total) return;
    float v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = 0.0f;
    for (int k = 0; k < splits; ++k) {
        float4 a = *reinterpret_cast<const float4 *>(part + (size_t)k * total + i);
        float4 b = *reinterpret_cast<const float4 *>(part + (size_t)k * total + i + 4);
        v[0] += a.x; v[1] += a.y; v[2] += a.z; v[3] += a.w;
        v[4] += b.x; v[5] += b.y; v[6] += b.z; v[7] += b.w;
    }
    const int co = (int)(i % Co);
    vec_t<bf16_t, 8> old, gt, r;
    if (is_grad && accum) old = *reinterpret_cast<const vec_t<bf16_t, 8> *>((old_from ? old_from : out) + i);
    if (is_grad && gate) gt = *reinterpret_cast<const vec_t<bf16_t, 8> *>(gate + i);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        float x = v[j] + (bias ? bias[co + j] : 0.0f);
        if (relu) x = fmaxf(x, 0.0f);
        r.e[j] = is_grad ? grad_out<bf16_t>(x, accum != 0, old.e[j], gate != nullptr, gt.e[j]) : from_f32<bf16_t>(x);
    }
    *reinterpret_cast<vec_t<bf16_t, 8> *>(out + i) = r;
}

struct GatherPlan {
    int bp, bc, splits, kt_per_split;
};

// Tile shape and split-K factor.  K is split only when there are very few output tiles (the linear
// layers: one pixel tile).
GatherPlan gather_plan(const GatherConv &g)
{
    GatherPlan p;
    const long long npix = (long long)g.N * g.Ho * g.Wo;
    p.bp = npix <= 64 ? 64 : 256;
    p.bc = g.Co <= 64 ? 64 : 128;
    if (p.bp == 64) p.bc = 128;
    auto tiles_of = [&](int bp) { return ((npix + bp - 1) / bp) * ((g.Co + p.bc - 1) / p.bc); };
    // 256-pixel tiles that cannot even fill 400 of the 512 block slots (14x14 layers, the 1x1 convs of
    // the bottleneck blocks): halve the pixel tile rather than split K, whose fp32 partials cost more
    // than the smaller tile loses (measured on 512-channel 14x14 layers: 73 us against 100 us)
    // Beside kernels of other streams the 196-392 tiles of 256 x 128 stay (measured on the deep VGG stage with three
    // streams: 18.8 -> 17.7 ms per mini-batch; alone on the chip the same choice loses 3 %).
    const bool few = g.beside && p.bp == 256 && p.bc == 128 && tiles_of(256) < 400 && tiles_of(256) >= 128;
    if (!few && p.bp == 256 && p.bc == 128 && tiles_of(256) < 400) p.bp = 128;
    // small products (the bottleneck blocks of ResNet: under ~8 GMAC) are bound by the latency of a block's
    // load - multiply - store chain, not by throughput: many 64-pixel blocks and no split of K were the
    // fastest choice on every such shape measured (e.g. 1x1 1024->256 at 14x14: 11.5 us against 22.2)
    if (p.bc == 128 && npix > 64 && (double)npix * g.Co * g.R * g.S * g.Ci < 8e9) p.bp = 64;
    // plenty of 256-pixel tiles and whole 256-channel tiles: one 8-wave block per CU owns 256 x 256, which
    // halves the L2 -> LDS traffic of two independent 256 x 128 blocks (3 % on the 512-channel 28x28 layers)
    if (!few && p.bp == 256 && p.bc == 128 && g.Co % 256 == 0) p.bc = 256;
    const long long tiles = tiles_of(p.bp);
    const int BK = 32;
    const int KT = g.Ci % BK == 0 ? (g.Ci / BK) * g.R * g.S : (g.R * g.S * g.Ci + BK - 1) / BK;
    long long want = tiles >= 128 ? 1 : (512 + tiles - 1) / tiles;
    long long most = KT / 16;                       // at least 16 K-tiles per split
    if (want > most) want = most;
    if (want > 32) want = 32;
    if (want < 1) want = 1;
    p.kt_per_split = (int)((KT + want - 1) / want);
    p.splits = (KT + p.kt_per_split - 1) / p.kt_per_split;
    return p;
}

template <int BP, int BC, int WP, int WC, int BK, int STAGES>
hipError_t launch_gather(const void *in, const void *wt, const float *bias, void *out, int relu, GradEpi epi,
                         const GatherConv &g, const GatherPlan &plan, void *workspace, hipStream_t s, bool raw = false,
                         float *stat_part = nullptr, const void *bn_x = nullptr, const float *bn_stats = nullptr)
{
    constexpr int NT = WP * WC * 64;
    constexpr size_t main_bytes = (size_t)STAGES * (BP + BC) * BK * 2;
    constexpr size_t epi_bytes = (size_t)BP * (BC + 4) * 2;
    constexpr size_t smem = (main_bytes > epi_bytes ? main_bytes : epi_bytes) + BC * sizeof(float);
    static_assert(smem <= (NT >= 512 ? 160 : 80) * 1024, "two blocks of 4 waves (one of 8) must fit the 160 KB LDS of a CU");
    const long long npix = (long long)g.N * g.Ho * g.Wo;
    const int tiles_p = (int)((npix + BP - 1) / BP), tiles_c = (g.Co + BC - 1) / BC;
    const int is_grad = (epi.gate != nullptr || epi.accum) ? 1 : 0;
    const unsigned in_bytes = (unsigned)((size_t)g.N * g.Hi * g.Wi * g.Ci * 2);
    const unsigned wt_bytes = (unsigned)((size_t)g.Co * g.R * g.S * g.Ci * 2);
    float *part = (plan.splits > 1 || raw) ? (float *)workspace : nullptr;      // raw: the fp32 partials are the result
    dim3 grid((unsigned)(tiles_p * tiles_c), (unsigned)plan.splits);
#define GATHER_LAUNCH(S1_, TI_)                                                                                   \
    do {                                                                                                          \
        auto kfn = k_gather_mfma<BP, BC, WP, WC, BK, STAGES, S1_, TI_>;                                           \
        static bool attr_set = false;                                                                             \
        if (!attr_set && smem > 64 * 1024) {                                                                      \
            hipError_t e = hipFuncSetAttribute((const void *)kfn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem); \
            if (e != hipSuccess) return e;                                                                        \
            attr_set = true;                                                                                      \
        }                                                                                                         \
        hipLaunchKernelGGL(kfn, grid, dim3(NT), smem, s, (const bf16_t *)in, (const bf16_t *)wt, bias,          \
                           (bf16_t *)out, (const bf16_t *)epi.gate, epi.accum, relu, is_grad, g, tiles_c, in_bytes, \
                           wt_bytes, part, plan.kt_per_split, stat_part, (const bf16_t *)bn_x, bn_stats,         \
                           (const bf16_t *)epi.accum_from);                                                      \
    } while (0)
    const bool taps_inner = g.Ci % BK == 0 && g.R * g.S <= 32;      // the stride-1 variant keeps a 32-bit tap mask
    if (g.s_in == 1) {
        if (taps_inner) GATHER_LAUNCH(true, true);
        else GATHER_LAUNCH(true, false);
    } else {
        if (taps_inner) GATHER_LAUNCH(false, true);
        else GATHER_LAUNCH(false, false);
    }
#undef GATHER_LAUNCH
    if (part && !raw) {
        const size_t total = (size_t)npix * g.Co;
        hipLaunchKernelGGL(k_gather_splitk_reduce, dim3((unsigned)((total / 8 + 255) / 256)), dim3(256), 0, s, part,
                           plan.splits, total, g.Co, bias, (bf16_t *)out, (const bf16_t *)epi.gate, epi.accum, relu,
                           is_grad, (const bf16_t *)epi.accum_from);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// wgrad
// ------------------------------------------------------------------------------------------
// The GEMM's N index is the flattened (r, s, c) filter position n = (r*S + s)*C + c, so a tile
// of BCI columns covers one tap (or part of it) when C >= BCI and several taps when C is small.
// grid: x = (ko tile, n tile) ; y = split over pixel chunks.  Same HBM -> LDS ring as the gather
// kernel: STAGES tiles of 32 pixels, requests issued STAGES-1 tiles ahead, hand-placed vmcnt waits.
template <int BKO, int BCI, int WKO, int WCI, int STAGES>
__global__ __launch_bounds__(WKO *WCI * 64, 2) void k_wgrad_mfma(const bf16_t *__restrict__ x,
                                                                  const bf16_t *__restrict__ dy,
                                                                  float *part, float *bpart, size_t split_stride,
                                                                  ConvShape c, int tiles_n, int pix_per_split,
                                                                  int add_to_dst, unsigned x_bytes,
                                                                  unsigned dy_bytes)
{
    constexpr int BKP = 32;
    constexpr int NW = WKO * WCI;
    constexpr int CPA = BKO / 8, CPB = BCI / 8;          // 16-byte chunks per tile row
    constexpr int AL = (BKP * CPA / 64) / NW, BL = (BKP * CPB / 64) / NW;   // wave-wide loads per wave and tile
    constexpr int WT_KO = BKO / WKO, WT_CI = BCI / WCI;
    constexpr int TA = WT_KO / 32, TB = WT_CI / 32;
    constexpr int STAGE_ELEMS = BKP * (BKO + BCI);
    constexpr unsigned OOB = 0x80000000u;
    static_assert(AL >= 1 && BL >= 1 && (BKP * CPA / 64) % NW == 0 && (BKP * CPB / 64) % NW == 0, "tile/thread mismatch");

    extern __shared__ __align__(16) unsigned char smem[];
    const lds_addr_of lds_of(smem);
    uint16_t *ring = reinterpret_cast<uint16_t *>(smem);         // [STAGES][ A tile | B tile ]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wk = wave % WKO, wi = wave / WKO;
    // The tiles of one pixel split read the same dy and x rows: number the blocks so that a split's tiles run on
    // one XCD (one L2) - consecutive block ids go round the eight XCDs, so each XCD gets a contiguous range of
    // (split, tile) positions.  With a single split (or few blocks) this is the identity up to a permutation.
    const int pos = xcd_remap((int)(blockIdx.y * gridDim.x + blockIdx.x), (int)(gridDim.x * gridDim.y));
    const int bx = pos % (int)gridDim.x, by = pos / (int)gridDim.x;
    const int tn = bx % tiles_n, tko = bx / tiles_n;
    const int ko0 = tko * BKO, n0 = tn * BCI;
    const int Ntot = c.R * c.S * c.C;
    const int npix = c.N * c.P * c.Q;
    const int p_begin = by * pix_per_split;
    const int p_end = p_begin + pix_per_split < npix ? p_begin + pix_per_split : npix;
    const int KT = (p_end - p_begin + BKP - 1) / BKP;

    __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(x), 0, (int)x_bytes, 0x00020000);
    __amdgpu_buffer_rsrc_t grsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(dy), 0, (int)dy_bytes, 0x00020000);

    // ---- A (dy) loads: lane fills slot (row, c') of wave-load q = i*NW + wave and fetches chunk c.
    // All addresses are kept as running byte offsets: a tile step adds a constant, so the loop body
    // has no multiplications.
    int ap[AL];                  // pixel of the lane's row in the current tile (huge if its chunk is past K)
    unsigned aoff[AL];           // byte offset of its chunk
#pragma unroll
    for (int i = 0; i < AL; ++i) {
        const int slot = (i * NW + wave) * 64 + lane;
        const int row = slot / CPA, cs = slot % CPA;
        const int ch = ((((cs >> 1) ^ wg_swz<BKO>(row)) << 1) | (cs & 1));
        const bool kin = ko0 + ch * 8 < c.K;
        ap[i] = kin ? p_begin + row : (1 << 30);
        aoff[i] = ((unsigned)(p_begin + row) * (unsigned)c.K + (unsigned)(ko0 + ch * 8)) * 2u;
    }
    // ---- B (x) loads: filter position of the lane's chunk column (fixed) and its pixel (advancing):
    // bp = output pixel index, (ph, pw) = stride * (output row, column), boff = byte offset of the
    // input element under the lane's tap.  Moving one output column / row / image forward changes
    // boff by a constant each.
    int bp[BL], ph[BL], pw[BL], br[BL], bs[BL];
    unsigned boff[BL];
    const int Qs = c.Q * c.stride, Ps = c.P * c.stride;
    const bool one_pixel = c.P == 1 && c.Q == 1;
    const unsigned sample_bytes = (unsigned)(c.H * c.W * c.C) * 2u;
    const unsigned colstep = (unsigned)(c.stride * c.C) * 2u;
    const unsigned rowstep = (unsigned)(c.stride * (c.W - c.Q) * c.C) * 2u;                 // extra, on top of Q columns
    const unsigned imgstep = (unsigned)((c.H - c.P * c.stride) * c.W * c.C) * 2u;           // extra, on top of P rows
#pragma unroll
    for (int i = 0; i < BL; ++i) {
        const int slot = (i * NW + wave) * 64 + lane;
        const int row = slot / CPB, cs = slot % CPB;
        const int ch = ((((cs >> 1) ^ wg_swz<BCI>(row)) << 1) | (cs & 1));
        const int n = n0 + ch * 8;
        const int tap = n / c.C, ci = n % c.C;
        br[i] = tap / c.S - c.pad;
        bs[i] = tap % c.S - c.pad;
        const int p0 = p_begin + row;
        bp[i] = n < Ntot ? p0 : (1 << 30);
        const int q = p0 % c.Q, t = p0 / c.Q;
        const int pr = t % c.P, img = t / c.P;
        ph[i] = pr * c.stride;
        pw[i] = q * c.stride;
        boff[i] = (unsigned)(((img * c.H + ph[i] + br[i]) * c.W + pw[i] + bs[i]) * c.C + ci) * 2u;   // may wrap at the borders
    }

    auto issue_tile = [&](int stage) {
        uint16_t *sa = ring + stage * STAGE_ELEMS, *sb = sa + BKP * BKO;
#pragma unroll
        for (int i = 0; i < AL; ++i) {
            unsigned vo = ap[i] < p_end ? aoff[i] : OOB;
            dma16(grsrc, lds_of(sa + (i * NW + wave) * 512), vo);
        }
#pragma unroll
        for (int i = 0; i < BL; ++i) {
            const bool ok = bp[i] < p_end && (unsigned)(ph[i] + br[i]) < (unsigned)c.H && (unsigned)(pw[i] + bs[i]) < (unsigned)c.W;
            unsigned vo = ok ? boff[i] : OOB;
            dma16(xrsrc, lds_of(sb + (i * NW + wave) * 512), vo);
        }
    };
    // step the per-lane pixel state to the next tile (kept out of issue_tile: its loops would split
    // the block in which the loads' address arithmetic interleaves with the MFMAs)
    auto advance_tile = [&]() {
#pragma unroll
        for (int i = 0; i < AL; ++i) {
            ap[i] += BKP;
            aoff[i] += (unsigned)(BKP * c.K) * 2u;
        }
#pragma unroll
        for (int i = 0; i < BL; ++i) {
            bp[i] += BKP;
            if (one_pixel) {                     // linear layers: every "pixel" is the next sample
                boff[i] += BKP * sample_bytes;
                continue;
            }
            pw[i] += BKP * c.stride;
            boff[i] += BKP * colstep;
            while (pw[i] >= Qs) {
                pw[i] -= Qs;
                boff[i] += rowstep;
                ph[i] += c.stride;
                if (ph[i] == Ps) {
                    ph[i] = 0;
                    boff[i] += imgstep;
                }
            }
        }
    };

    f32x16_t acc[TA][TB];
#pragma unroll
    for (int a = 0; a < TA; ++a)
#pragma unroll
        for (int b = 0; b < TB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;

    // bias gradient = column sums of dy: the waves holding the dy fragments of filter-column tile 0
    // add up their fragment values on the side (lane -> output channel, 8 pixels per step)
    const bool do_bias = bpart != nullptr && tn == 0 && wi == 0;
    float bsum[TA];
#pragma unroll
    for (int a = 0; a < TA; ++a) bsum[a] = 0.0f;

    auto load_frags = [&](int stage, int k0, bf16x8_t(&fa)[TA], bf16x8_t(&fb)[TB]) {
        const uint16_t *sa = ring + stage * STAGE_ELEMS, *sb = sa + BKP * BKO;
#pragma unroll
        for (int a = 0; a < TA; ++a) fa[a] = tr_frag<BKO>(sa, wk * WT_KO + a * 32, k0, lane);
#pragma unroll
        for (int b = 0; b < TB; ++b) fb[b] = tr_frag<BCI>(sb, wi * WT_CI + b * 32, k0, lane);
    };
    auto mfma_all = [&](const bf16x8_t(&fa)[TA], const bf16x8_t(&fb)[TB]) {
        if (do_bias) {
#pragma unroll
            for (int a = 0; a < TA; ++a) bsum[a] = frag_sum(fa[a], bsum[a]);
        }
#pragma unroll
        for (int a = 0; a < TA; ++a)
#pragma unroll
            for (int b = 0; b < TB; ++b)
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
    };

    // Same software pipeline as the gather kernel: STAGES tiles in the ring, fragments double-buffered
    // in registers, the barrier that publishes tile kt+1 between the two MFMA groups of tile kt.
    constexpr int NLOAD = AL + BL;
#pragma unroll
    for (int st = 0; st < STAGES; ++st) {
        issue_tile(st);
        advance_tile();
    }
    WAIT_VMCNT((STAGES - 1) * NLOAD);
    WAIT_LGKMCNT(0);
    __builtin_amdgcn_s_barrier();
    bf16x8_t fa0[TA], fb0[TB], fa1[TA], fb1[TB];
    load_frags(0, 0, fa0, fb0);
    int rd = 0;
    for (int kt = 0; kt < KT; ++kt) {
        const int nx = rd + 1 == STAGES ? 0 : rd + 1;
        load_frags(rd, 16, fa1, fb1);
        __builtin_amdgcn_sched_barrier(0);
        mfma_all(fa0, fb0);
        __builtin_amdgcn_sched_barrier(0);
        WAIT_LGKMCNT(0);
        WAIT_VMCNT((STAGES - 2) * NLOAD);
        __builtin_amdgcn_s_barrier();
        load_frags(nx, 0, fa0, fb0);
        __builtin_amdgcn_sched_barrier(0);
        issue_tile(rd);
        mfma_all(fa1, fb1);
        __builtin_amdgcn_sched_barrier(0);
        advance_tile();
        rd = nx;
    }
    WAIT_VMCNT(0);

    // partial[split][ko][n]
    float *dst = part + (size_t)by * split_stride;
    const int col = lane & 31, half = lane >> 5;
    if (do_bias) {
        float *bdst = bpart + (size_t)by * split_stride;
#pragma unroll
        for (int a = 0; a < TA; ++a) {
            const float t = bsum[a] + __shfl_xor(bsum[a], 32, 64);
            const int ko = ko0 + wk * WT_KO + a * 32 + col;
            if (half == 0 && ko < c.K) bdst[ko] = add_to_dst ? bdst[ko] + t : t;
        }
    }
    // The accumulators leave through LDS: each wave parks one 32-row slice of its sub-tile in a region
    // of its own ([32][WT_CI] floats; the ring is free by now) and reads it back as float4 so that 16
    // lanes cover 256 contiguous bytes of one dw row.  Straight from the registers a row segment would
    // be 32 separate 4-byte read-modify-writes.
    __syncthreads();                                          // every wave has left the ring
    float *stg = reinterpret_cast<float *>(smem) + wave * (32 * WT_CI);
    constexpr int F4R = WT_CI / 4;                            // float4 per staged row
    constexpr int RPI = 64 / F4R;                             // rows one wave-wide access covers
#pragma unroll
    for (int a = 0; a < TA; ++a) {
#pragma unroll
        for (int b = 0; b < TB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) stg[(8 * (v >> 2) + 4 * half + (v & 3)) * WT_CI + b * 32 + col] = acc[a][b][v];
        WAIT_LGKMCNT(0);
        __builtin_amdgcn_wave_barrier();
        // all reads of the slice first, then all writes: one round trip to memory per slice, not one per row group
        constexpr int IT = 32 / RPI;
        float4 t[IT], o[IT];
#pragma unroll
        for (int it = 0; it < IT; ++it) {
            const int row = it * RPI + lane / F4R, c4 = (lane % F4R) * 4;
            const int ko = ko0 + wk * WT_KO + a * 32 + row, n = n0 + wi * WT_CI + c4;
            t[it] = *reinterpret_cast<const float4 *>(stg + row * WT_CI + c4);
            o[it] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (add_to_dst && ko < c.K && n < Ntot) o[it] = *reinterpret_cast<const float4 *>(dst + (size_t)ko * Ntot + n);
        }
#pragma unroll
        for (int it = 0; it < IT; ++it) {
            const int row = it * RPI + lane / F4R, c4 = (lane % F4R) * 4;
            const int ko = ko0 + wk * WT_KO + a * 32 + row, n = n0 + wi * WT_CI + c4;
            if (ko < c.K && n < Ntot)
                *reinterpret_cast<float4 *>(dst + (size_t)ko * Ntot + n) =
                    make_float4(t[it].x + o[it].x, t[it].y + o[it].y, t[it].z + o[it].z, t[it].w + o[it].w);
        }
        WAIT_LGKMCNT(0);
        __builtin_amdgcn_wave_barrier();
    }
}

// dw[i] += sum_k part[k][i].  A block owns 64 float4 columns; its 4 split-lanes walk the partials
// with stride 4 and are combined through LDS in lane order (the result does not depend on timing).
// Entries past total_w are the bias partials and go to db.  total_w and total are multiples of 4
// (channel counts are multiples of 8).
__global__ void k_splitk_reduce(const float *__restrict__ part, float *dw, float *db, size_t total_w, size_t total,
                                int splits)
{
    __shared__ float4 red[4][64];
    const int col = threadIdx.x & 63, sl = threadIdx.x >> 6;
    const size_t i = ((size_t)blockIdx.x * 64 + col) * 4;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i < total) {
#pragma unroll 4
        for (int k = sl; k < splits; k += 4) {
            float4 v = *reinterpret_cast<const float4 *>(part + (size_t)k * total + i);
            acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
        }
    }
    red[sl][col] = acc;
    __syncthreads();
    if (sl == 0 && i < total) {
        float *out = i < total_w ? dw + i : db + (i - total_w);
        float4 d = *reinterpret_cast<float4 *>(out);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            float4 v = red[k][col];
            d.x += v.x; d.y += v.y; d.z += v.z; d.w += v.w;
        }
        *reinterpret_cast<float4 *>(out) = d;
    }
}

struct WgradPlan {
    int bko, bci, tiles_ko, tiles_n, splits, pix_per_split;
};

WgradPlan wgrad_plan(const ConvShape &c)
{
    WgradPlan p;
    const int Ntot = c.R * c.S * c.C;
    p.bko = c.K > 128 ? 256 : (c.K > 64 ? 128 : 64);
    p.bci = Ntot > 64 ? 128 : 64;
    if (p.bko == 256 && p.bci == 64) p.bko = 128;
    // small products (under ~8 GMAC, the bottleneck blocks of ResNet) are latency-bound: more, smaller
    // tiles measured 10-25 % faster than 256-wide ones on every such shape
    if (p.bko == 256 && (double)c.N * c.P * c.Q * c.K * Ntot < 8e9) p.bko = 128;
    p.tiles_ko = (c.K + p.bko - 1) / p.bko;
    p.tiles_n = (Ntot + p.bci - 1) / p.bci;
    long long npix = (long long)c.N * c.P * c.Q;
    long long tiles = (long long)p.tiles_ko * p.tiles_n;
    // Split count: the chip holds 512 blocks at once (256 CUs x 2), and a launch whose block count is
    // just above a multiple of that leaves most CUs idle during the last blocks.  Take the split count
    // that minimises (time relative to perfectly filled rounds) + (relative cost of the partials: every
    // split writes and re-reads a full fp32 copy of dw, about 500/npix of the MFMA time each); at least
    // 512 pixels per split.
    long long max_by_work = (npix + 511) / 512;
    if (max_by_work > 256) max_by_work = 256;
    if (max_by_work < 1) max_by_work = 1;
    const long long slots = 512;
    long long want = 1;
    double best = 1e30;
    for (long long sp = 1; sp <= max_by_work; ++sp) {
        const long long blocks = tiles * sp, rounds = (blocks + slots - 1) / slots;
        const double cost = (double)(rounds * slots) / (double)blocks + 500.0 * (double)sp / (double)npix;
        if (cost < best) {
            best = cost;
            want = sp;
        }
    }
    long long pps = (npix + want - 1) / want;
    pps = (pps + 31) / 32 * 32;
    if (pps < 32) pps = 32;
    p.pix_per_split = (int)pps;
    p.splits = (int)((npix + pps - 1) / pps);
    if (p.splits < 1) p.splits = 1;
    return p;
}

}  // namespace

bool conv_gather_mfma_supported(const GatherConv &g)
{
    // byte offsets into the operands are 32-bit (buffer addressing)
    return g.Ci % 8 == 0 && g.Co % 8 == 0 && g.Ci >= 8 && g.s_in >= 1 && g.s_out >= 1 &&
           (long long)g.N * g.Hi * g.Wi * g.Ci * 2 < (1ll << 31) && (long long)g.Co * g.R * g.S * g.Ci * 2 < (1ll << 31) &&
           (long long)g.N * g.Ho * g.Wo < (1ll << 31) - 512;
}

size_t conv_gather_mfma_workspace(const GatherConv &g)
{
    if (conv3x3_halo_supported(g) || conv3x3_c8_supported(g)) return 0;
    GatherPlan p = gather_plan(g);
    return p.splits > 1 ? (size_t)p.splits * g.N * g.Ho * g.Wo * g.Co * sizeof(float) : 0;
}

int conv_gather_mfma_stat_chunks(const GatherConv &g)
{
    if (!conv_gather_mfma_supported(g) || conv3x3_halo_supported(g) || conv3x3_c8_supported(g)) return 0;
    const GatherPlan p = gather_plan(g);
    if (p.splits != 1) return 0;
    return (int)(((long long)g.N * g.Ho * g.Wo + p.bp - 1) / p.bp);
}

hipError_t conv_gather_mfma(const void *in, const void *wt, const float *bias, void *out, int relu,
                            GradEpi epi, const GatherConv &g, void *workspace, hipStream_t s, float *stat_part,
                            const void *bn_x, const float *bn_stats)
{
    if (!conv_gather_mfma_supported(g)) return hipErrorInvalidValue;
    if (stat_part && conv_gather_mfma_stat_chunks(g) == 0) return hipErrorInvalidValue;
    if (bn_x && (!stat_part || !bn_stats || !(epi.gate || epi.accum))) return hipErrorInvalidValue;   // gradient epilogue only
    if ((long long)g.N * g.Ho * g.Wo == 0) return hipSuccess;
    if (epi.accum_from && (!epi.accum || conv3x3_halo_supported(g))) return hipErrorInvalidValue;   // gather kernel only
    if (conv3x3_halo_supported(g)) return conv3x3_halo_mfma(in, wt, bias, out, relu, epi, g, s);
    if (!epi.gate && !epi.accum && conv3x3_c8_supported(g)) return conv3x3_c8_mfma(in, wt, bias, out, relu, g, s);
    const GatherPlan p = gather_plan(g);
    if (p.bp == 64) return launch_gather<64, 128, 1, 4, 32, 3>(in, wt, bias, out, relu, epi, g, p, workspace, s, false, stat_part, bn_x, bn_stats);
    if (p.bc == 64) return launch_gather<256, 64, 4, 1, 32, 3>(in, wt, bias, out, relu, epi, g, p, workspace, s, false, stat_part, bn_x, bn_stats);
    if (p.bc == 256) return launch_gather<256, 256, 2, 4, 32, 3>(in, wt, bias, out, relu, epi, g, p, workspace, s, false, stat_part, bn_x, bn_stats);
    if (p.bp == 128) return launch_gather<128, 128, 2, 2, 32, 3>(in, wt, bias, out, relu, epi, g, p, workspace, s, false, stat_part, bn_x, bn_stats);
    return launch_gather<256, 128, 2, 2, 32, 3>(in, wt, bias, out, relu, epi, g, p, workspace, s, false, stat_part, bn_x, bn_stats);
}

size_t conv_gather_mfma_raw_workspace(const GatherConv &g)
{
    return (size_t)gather_plan(g).splits * g.N * g.Ho * g.Wo * g.Co * sizeof(float);
}

hipError_t conv_gather_mfma_raw(const void *in, const void *wt, const GatherConv &g, float *part, int *splits,
                                hipStream_t s)
{
    if (!conv_gather_mfma_supported(g) || !part || !splits || g.Co % 4 != 0) return hipErrorInvalidValue;
    const GatherPlan p = gather_plan(g);
    *splits = p.splits;
    if ((long long)g.N * g.Ho * g.Wo == 0) return hipSuccess;
    const GradEpi none{nullptr, 0};
    if (p.bp == 64) return launch_gather<64, 128, 1, 4, 32, 3>(in, wt, nullptr, nullptr, 0, none, g, p, part, s, true);
    if (p.bc == 64) return launch_gather<256, 64, 4, 1, 32, 3>(in, wt, nullptr, nullptr, 0, none, g, p, part, s, true);
    if (p.bc == 256) return launch_gather<256, 256, 2, 4, 32, 3>(in, wt, nullptr, nullptr, 0, none, g, p, part, s, true);
    if (p.bp == 128) return launch_gather<128, 128, 2, 2, 32, 3>(in, wt, nullptr, nullptr, 0, none, g, p, part, s, true);
    return launch_gather<256, 128, 2, 2, 32, 3>(in, wt, nullptr, nullptr, 0, none, g, p, part, s, true);
}

bool conv_wgrad_mfma_supported(const ConvShape &c)
{
    // 32-bit byte offsets into both operands (buffer addressing)
    return c.C % 8 == 0 && c.K % 8 == 0 && c.C >= 8 && c.K >= 8 &&
           (long long)c.N * c.H * c.W * c.C * 2 < (1ll << 31) && (long long)c.N * c.P * c.Q * c.K * 2 < (1ll << 31);
}

size_t conv_wgrad_mfma_workspace(const ConvShape &c)
{
    if (wgrad3x3_halo_supported(c)) return wgrad3x3_halo_workspace(c);
    if (wgrad3x3_c8_supported(c)) return wgrad3x3_c8_workspace(c);
    WgradPlan p = wgrad_plan(c);
    return p.splits == 1 ? 0 : (size_t)p.splits * ((size_t)c.K * c.R * c.S * c.C + c.K) * sizeof(float);
}

hipError_t conv_wgrad_mfma(const void *x, const void *dy, float *dw, float *db, void *workspace,
                           const ConvShape &c, hipStream_t s)
{
    if (!conv_wgrad_mfma_supported(c)) return hipErrorInvalidValue;
    if ((long long)c.N * c.P * c.Q == 0) return hipSuccess;
    if (wgrad3x3_halo_supported(c)) return wgrad3x3_halo_mfma(x, dy, dw, db, workspace, c, s);
    if (wgrad3x3_c8_supported(c)) return wgrad3x3_c8_mfma(x, dy, dw, db, workspace, c, s);
    WgradPlan p = wgrad_plan(c);
    dim3 grid((unsigned)(p.tiles_ko * p.tiles_n), (unsigned)p.splits);
    const int direct = p.splits == 1;
    const size_t total_w = (size_t)c.K * c.R * c.S * c.C, total = total_w + (db ? c.K : 0);
    float *part = direct ? dw : (float *)workspace;
    float *bpart = !db ? nullptr : (direct ? db : part + total_w);
#define WG_LAUNCH(BKO_, BCI_, WKO_, WCI_)                                                                  \
    do {                                                                                                   \
        constexpr size_t smem = (size_t)3 * 32 * (BKO_ + BCI_) * 2;                                        \
        auto kfn = k_wgrad_mfma<BKO_, BCI_, WKO_, WCI_, 3>;                                                \
        static bool attr_set = false;                                                                      \
        if (!attr_set && smem > 64 * 1024) {                                                               \
            hipError_t e = hipFuncSetAttribute((const void *)kfn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem); \
            if (e != hipSuccess) return e;                                                                 \
            attr_set = true;                                                                               \
        }                                                                                                  \
        hipLaunchKernelGGL(kfn, grid, dim3(WKO_ * WCI_ * 64), smem, s, (const bf16_t *)x, (const bf16_t *)dy, part, bpart, \
                           total, c, p.tiles_n, p.pix_per_split, direct, x_bytes, dy_bytes);               \
    } while (0)
    const unsigned x_bytes = (unsigned)((size_t)c.N * c.H * c.W * c.C * 2);
    const unsigned dy_bytes = (unsigned)((size_t)c.N * c.P * c.Q * c.K * 2);
    if (p.bko == 256)
        WG_LAUNCH(256, 128, 2, 2);
    else if (p.bko == 128 && p.bci == 128)
        WG_LAUNCH(128, 128, 2, 2);
    else if (p.bko == 64 && p.bci == 128)
        WG_LAUNCH(64, 128, 1, 4);
    else if (p.bko == 128 && p.bci == 64)
        WG_LAUNCH(128, 64, 4, 1);
    else
        WG_LAUNCH(64, 64, 2, 2);
#undef WG_LAUNCH
    if (!direct)
        hipLaunchKernelGGL(k_splitk_reduce, dim3((unsigned)((total / 4 + 63) / 64)), dim3(256), 0, s, part,
                           dw, db, total_w, total, p.splits);
    return hipGetLastError();
}

}  // namespace bapipe
