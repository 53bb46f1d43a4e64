// 3x3 / stride 1 / pad 1 convolution (forward, and dgrad through the flipped filter) for feature
// maps whose sides are multiples of 16: the layers of the first VGG stage (224x224 and 112x112,
// 64 / 128 channels), where the generic gather kernel is bound by L1/L2 traffic because every
// input pixel is fetched again for each of the 9 taps.
//
// A block owns a 16x16 patch of output pixels x 64 output channels.  The 18x18 input halo of one
// 64-channel slice is brought into LDS ONCE (buffer_load ... lds, zero fill outside the image) and
// all 9 taps read their shifted views of it: the B fragment of tap (r,s) for patch pixel (y,x) is
// simply halo pixel (y+r, x+s).  Only the filter tile of the current tap streams through a small
// LDS ring.  HBM/L2 traffic per output drops from 9 input reads to (18*18)/(16*16) = 1.27.
// MFMA mapping, swizzles and the epilogue are those of the gather kernel (A = filter rows, B = pixels,
// v_mfma_f32_32x32x16_bf16, staging through LDS to 16-byte coalesced rows).
#include "kernels.h"
#include "mfma_common.h"

namespace bapipe {
namespace {

// rows of 64 bf16 (8 chunks of 16 bytes): 16 consecutive rows read the same chunk column without
// bank conflicts when the chunk index is XORed with bits 1..3 of the row
__device__ __forceinline__ int swz8(int row) { return (row >> 1) & 7; }

constexpr int PATCH = 16, HALO = 18, HPIX = HALO * HALO;       // 324 halo pixels
constexpr int HL = 11;                                          // halo wave-loads per wave (44 x 64 slots >= 2592)
// A block's tile is 64 output channels wide, whatever the layer's width (a 128-channel layer is two tiles that
// load the same halo): filter steps of 32 input channels (4 KB stages) through a ring of two, and exactly the 41
// wave-loads that hold halo pixels, so that a block needs 50.4 KB of LDS (40 allocation granules of 1280 bytes)
// and at most 168 registers and THREE blocks share a CU.  A block has little arithmetic per byte it moves (one
// 64-channel slice per halo), spends much of its life fetching its halo and storing its patch, and the third
// block is what overlaps that.  128-channel tiles (128 accumulator registers per lane, two blocks per CU) were the
// first design for the 128-channel layers and lost to this one once it had its third block: whole first VGG stage
// on one stream 9.90 -> 9.41 ms per mini-batch.  Measured on the 64 -> 64 layer at 224 x 224 against two blocks
// per CU: forward 171 -> 155 us, forward + pool 180 -> 142 us, input gradient 240 -> 207 us.
struct halo_cfg {
    static constexpr int BC = 64;                                  // output channels per block
    static constexpr int KS = 32;                                  // input channels per filter step
    static constexpr int WS = 2;                                   // ring stages
    static constexpr int LOADS = 41;                               // wave-loads that hold halo pixels (41 x 64 slots >= 2592)
    static constexpr int ELEMS = LOADS * 64 * 8;                   // bf16 elements reserved for the halo tile
    static constexpr int BLOCKS_PER_CU = 3;
};

// Filter tiles stream through the ring: one "step" is one tap x KS = 32 input channels, i.e. NSUB = 2 MFMA
// sub-steps, and a stage holds BC x 32 filter values.  The taps of a slice are
// unrolled, so ring slots, halo rows and swizzles are compile-time or precomputed per tap: a fragment
// read costs at most one XOR.  Fragments are double-buffered in registers and the barrier that
// publishes the next filter tile sits before the last sub-step of a step, as in the gather kernel.
__global__ __launch_bounds__(256, halo_cfg::BLOCKS_PER_CU) void k_conv3x3_halo(const bf16_t *__restrict__ in, const bf16_t *__restrict__ wt,
                                                         const float *__restrict__ bias, bf16_t *out,
                                                         const bf16_t *__restrict__ gate, int accum, int relu,
                                                         int is_grad, int N, int H, int W, int Ci, int Co,
                                                         unsigned in_bytes, unsigned wt_bytes,
                                                         bf16_t *__restrict__ pool_out, uint8_t *__restrict__ pool_idx)
{
    constexpr int NW = 4, BC = halo_cfg::BC;
    constexpr int KS = halo_cfg::KS;           // input channels per filter step tile
    constexpr int HALO_LOADS = halo_cfg::LOADS, HALO_ELEMS = halo_cfg::ELEMS;
    constexpr int NSUB = KS / 16;              // MFMA sub-steps per step
    constexpr int SPT = 64 / KS;               // steps per tap and 64-channel slice
    constexpr int SPS = 9 * SPT;               // steps per slice (a multiple of WS)
    constexpr int WS = halo_cfg::WS;           // ring stages
    constexpr int WT_ELEMS = BC * KS;          // 2048 elements = 4 KB
    constexpr int CPR = KS / 8;                // 16-byte chunks per filter-tile row
    constexpr int WLD = WT_ELEMS / 8 / 256;    // filter wave-loads per wave and step (256 slots / 64 / 4)
    constexpr int TC = BC / 32, TP = 2;        // wave tile: BC channels x 64 pixels
    constexpr int SROW = BC + 4;
    constexpr unsigned OOB = 0x80000000u;
    static_assert(WT_ELEMS == 2048 && KS == 32 && SPS % WS == 0, "ring layout");

    extern __shared__ __align__(16) unsigned char smem[];
    const lds_addr_of lds_of(smem);
    uint16_t *halo = reinterpret_cast<uint16_t *>(smem);
    uint16_t *wring = halo + HALO_ELEMS;
    uint16_t *sO = reinterpret_cast<uint16_t *>(smem);                                   // [256][SROW] (epilogue)
    float *sBias = reinterpret_cast<float *>(smem + (size_t)(HALO_ELEMS + WS * WT_ELEMS) * 2);   // [BC]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tiles_c = Co / BC, px_tiles = W / PATCH, py_tiles = H / PATCH;
    const int bid = xcd_remap(blockIdx.x, gridDim.x);
    const int tile_c = bid % tiles_c;
    int t = bid / tiles_c;
    const int X0 = (t % px_tiles) * PATCH;
    t /= px_tiles;
    const int Y0 = (t % py_tiles) * PATCH;
    const int n = t / py_tiles;
    const int co0 = tile_c * BC;
    const int NS = Ci / 64;

    __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(in), 0, (int)in_bytes, 0x00020000);
    __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(wt), 0, (int)wt_bytes, 0x00020000);

    // halo slot of a lane: slot = hr*8 + c', it fetches chunk c = c' ^ swz8(hr) of halo pixel hr (offsets
    // are recomputed per slice: keeping 11 of them alive through the main loop costs more than that)
    auto issue_halo = [&](int slice) {
#pragma unroll
        for (int i = 0; i < HL; ++i) {
            const int slot = (i * NW + wave) * 64 + lane;
            const int hr = slot >> 3, c = (slot & 7) ^ swz8(hr);
            const int hy = hr / HALO, hx = hr - hy * HALO;
            const int y = Y0 - 1 + hy, x = X0 - 1 + hx;
            const bool ok = hr < HPIX && (unsigned)y < (unsigned)H && (unsigned)x < (unsigned)W;
            unsigned vo = ok ? ((unsigned)((n * H + y) * W + x) * (unsigned)Ci + (unsigned)(slice * 64 + c * 8)) * 2u : OOB;
            if (i * NW + wave < HALO_LOADS) dma16(xrsrc, lds_of(halo + (i * NW + wave) * 512), vo);
        }
    };
    // filter tile rows are KS = 32 elements long; chunk index XORed with bits 2..3 of the row so that the
    // fragment reads are conflict free
    auto wswz = [](int row) { return (row >> 2) & 3; };
    unsigned woff[WLD];
#pragma unroll
    for (int i = 0; i < WLD; ++i) {
        const int slot = (i * NW + wave) * 64 + lane;
        const int row = slot / CPR, c = (slot % CPR) ^ wswz(row);
        woff[i] = ((unsigned)(co0 + row) * 9u * (unsigned)Ci + (unsigned)c * 8u) * 2u;
    }
    const unsigned wring_addr = lds_of(wring);
    auto issue_w = [&](int slice, int pos) {        // step `pos` (= tap*SPT + half) of a slice
        const int tap = pos / SPT, half = pos % SPT;
        const unsigned ko = slice < NS ? (unsigned)(tap * Ci + slice * 64 + half * KS) * 2u : OOB;
#pragma unroll
        for (int i = 0; i < WLD; ++i)
            dma16(wrsrc, wring_addr + (unsigned)((pos % WS) * WT_ELEMS * 2 + (i * NW + wave) * 1024), (woff[i] + ko) | (ko & OOB));
    };

    f32x16_t acc[TC][TP];
#pragma unroll
    for (int a = 0; a < TC; ++a)
#pragma unroll
        for (int b = 0; b < TP; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;

    const int frow = lane & 31, fhalf = lane >> 5;
    const int py = 4 * wave + (frow >> 4), px = frow & 15;       // patch pixel of B tile 0 (tile 1: py + 2)

    // fragment addresses (bytes).  The K position of a sub-step only flips bits 5..6 (the chunk pair),
    // which commutes with the swizzle XOR: address(kk) = base ^ (kk << 5).
    unsigned hbase[9][TP];
#pragma unroll
    for (int tap = 0; tap < 9; ++tap)
#pragma unroll
        for (int b = 0; b < TP; ++b) {
            const int hr = (py + tap / 3 + 2 * b) * HALO + px + tap % 3;
            hbase[tap][b] = (unsigned)(hr * 128 + ((fhalf ^ swz8(hr)) << 4));
        }
    unsigned wbase[TC];
#pragma unroll
    for (int a = 0; a < TC; ++a) {
        const int row = a * 32 + frow;
        wbase[a] = (unsigned)(HALO_ELEMS * 2 + row * KS * 2 + ((fhalf ^ wswz(row)) << 4));
    }
    auto load_frags = [&](int pos, int ks, bf16x8_t(&fa)[TC], bf16x8_t(&fb)[TP]) {
        const int tap = pos / SPT, half = pos % SPT;
#pragma unroll
        for (int a = 0; a < TC; ++a)
            fa[a] = as_frag(*reinterpret_cast<const chunk16 *>(smem + (wbase[a] ^ (unsigned)(ks << 5)) + (pos % WS) * WT_ELEMS * 2));
#pragma unroll
        for (int b = 0; b < TP; ++b)
            fb[b] = as_frag(*reinterpret_cast<const chunk16 *>(smem + (hbase[tap][b] ^ (unsigned)((half * NSUB + ks) << 5))));
    };
    auto mfma_all = [&](const bf16x8_t(&fa)[TC], const bf16x8_t(&fb)[TP]) {
#pragma unroll
        for (int a = 0; a < TC; ++a)
#pragma unroll
            for (int b = 0; b < TP; ++b)
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
    };

    if (tid < BC) sBias[tid] = bias ? bias[co0 + tid] : 0.0f;          // read after the main loop's barriers

    issue_halo(0);
#pragma unroll
    for (int st = 0; st < WS; ++st) issue_w(0, st);

    constexpr int CH8 = BC / 8;
    constexpr int UNITS = 256 * CH8 / 256;
    const chunk16 zero16 = {0u, 0u, 0u, 0u};
    WAIT_VMCNT((WS - 1) * WLD);                  // halo and filter tile 0 have landed
    WAIT_LGKMCNT(0);                             // no scalar load pending at loop entry (else every LDS wait is a full drain)
    __builtin_amdgcn_s_barrier();
    bf16x8_t fa0[TC], fb0[TP], fa1[TC], fb1[TP];
    load_frags(0, 0, fa0, fb0);
    for (int slice = 0; slice < NS; ++slice) {
        // keep the 26 base addresses opaque per slice: otherwise all 80 XORed fragment addresses are
        // hoisted out of this loop and spill
#pragma unroll
        for (int tap = 0; tap < 9; ++tap)
#pragma unroll
            for (int b = 0; b < TP; ++b) asm volatile("" : "+v"(hbase[tap][b]));
#pragma unroll
        for (int a = 0; a < TC; ++a) asm volatile("" : "+v"(wbase[a]));
#pragma unroll
        for (int pos = 0; pos < SPS; ++pos) {
            // sub-steps 0 .. NSUB-2: fetch the next sub-step's fragments, multiply the current ones
#pragma unroll
            for (int ks = 0; ks + 1 < NSUB; ++ks) {
                if (ks % 2 == 0) {
                    load_frags(pos, ks + 1, fa1, fb1);
                    __builtin_amdgcn_sched_barrier(0);
                    mfma_all(fa0, fb0);
                } else {
                    load_frags(pos, ks + 1, fa0, fb0);
                    __builtin_amdgcn_sched_barrier(0);
                    mfma_all(fa1, fb1);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            // last sub-step (its fragments are in fa1/fb1: NSUB is even): publish the next filter tile first
            WAIT_LGKMCNT(0);                          // this wave has read everything it needs from this step's tile
            WAIT_VMCNT((WS - 2) * WLD);
            __builtin_amdgcn_s_barrier();
            if (pos + 1 < SPS) {
                load_frags(pos + 1, 0, fa0, fb0);
                __builtin_amdgcn_sched_barrier(0);
                if (pos + WS < SPS)
                    issue_w(slice, pos + WS);
                else
                    issue_w(slice + 1, pos + WS - SPS);
                mfma_all(fa1, fb1);
                __builtin_amdgcn_sched_barrier(0);
            } else {
                // slice boundary: every wave has left the halo, bring in the next 64 input channels
                if (slice + 1 < NS) issue_halo(slice + 1);
                issue_w(slice + 1, pos + WS - SPS);
                mfma_all(fa1, fb1);
                __builtin_amdgcn_sched_barrier(0);
                WAIT_VMCNT(0);
                __builtin_amdgcn_s_barrier();
                load_frags(0, 0, fa0, fb0);
            }
        }
    }
    WAIT_VMCNT(0);
    __syncthreads();

    // gradient epilogue: the ReLU-gate rows are requested here, after the last MFMA (the main loop has no registers to
    // spare for an earlier request), so that they travel while the accumulators are parked in the staging tile
    chunk16 glate[UNITS];
    if (is_grad && gate) {
#pragma unroll
        for (int it = 0; it < UNITS; ++it) {
            const int u = tid + it * 256;
            const int pj = u / CH8, c8i = u % CH8;
            const size_t p = (size_t)(n * H + Y0 + (pj >> 4)) * W + X0 + (pj & 15);
            glate[it] = *reinterpret_cast<const chunk16 *>(gate + p * Co + co0 + c8i * 8);
        }
    }

    // ---- epilogue: every wave parks its 64 pixels x BC channels in LDS (bf16, bias / ReLU applied),
    // one barrier, then the block streams the patch out as 16-byte coalesced rows
#pragma unroll
    for (int a = 0; a < TC; ++a) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int col = a * 32 + 8 * q + 4 * fhalf;
            const float4 bv = *reinterpret_cast<const float4 *>(sBias + col);
#pragma unroll
            for (int b = 0; b < TP; ++b) {
                const int prow = wave * 64 + b * 32 + frow;
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
    __syncthreads();
    if (pool_out) {
        // fused 2x2 stride-2 max-pool: the patch holds 8x8 complete windows; the conv output itself
        // never reaches memory.  Window scan order and tie rule (first maximum) are those of the
        // stand-alone pooling kernel.
        const int Hq = H / 2, Wq = W / 2;
#pragma unroll
        for (int it = 0; it < 64 * CH8 / 256; ++it) {
            const int u = tid + it * 256;
            const int qp = u / CH8, c8i = u % CH8;
            const int qy = qp >> 3, qx = qp & 7;
            uint32_t w[4][4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int pj = (2 * qy + (k >> 1)) * 16 + 2 * qx + (k & 1);
                const chunk8 lo = *reinterpret_cast<const chunk8 *>(sO + pj * SROW + c8i * 8);
                const chunk8 hi = *reinterpret_cast<const chunk8 *>(sO + pj * SROW + c8i * 8 + 4);
                w[k][0] = lo[0]; w[k][1] = lo[1]; w[k][2] = hi[0]; w[k][3] = hi[1];
            }
            chunk16 best;
            chunk8 bidx = {0u, 0u};
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int sh = 16 * (j & 1);
                uint32_t bv = (w[0][j >> 1] >> sh) & 0xFFFFu;
                uint32_t bi = 0;
#pragma unroll
                for (int k = 1; k < 4; ++k) {
                    const uint32_t v = (w[k][j >> 1] >> sh) & 0xFFFFu;
                    if (__uint_as_float(v << 16) > __uint_as_float(bv << 16)) {       // strictly greater: the first maximum wins
                        bv = v;
                        bi = (uint32_t)k;
                    }
                }
                if (j & 1)
                    best[j >> 1] |= bv << 16;
                else
                    best[j >> 1] = bv;
                bidx[j >> 2] |= bi << (8 * (j & 3));
            }
            const size_t q = ((size_t)(n * Hq + Y0 / 2 + qy) * Wq + X0 / 2 + qx) * Co + co0 + c8i * 8;
            *reinterpret_cast<chunk16 *>(pool_out + q) = best;
            *reinterpret_cast<chunk8 *>(pool_idx + q) = bidx;
        }
        return;
    }
#pragma unroll
    for (int it = 0; it < UNITS; ++it) {
        const int u = tid + it * 256;
        const int pj = u / CH8, c8i = u % CH8;
        const size_t p = (size_t)(n * H + Y0 + (pj >> 4)) * W + X0 + (pj & 15);
        const int co = co0 + c8i * 8;
        chunk8 lo = *reinterpret_cast<const chunk8 *>(sO + pj * SROW + c8i * 8);
        chunk8 hi = *reinterpret_cast<const chunk8 *>(sO + pj * SROW + c8i * 8 + 4);
        chunk16 v = {lo[0], lo[1], hi[0], hi[1]};
        bf16_t *dst = out + p * Co + co;
        if (is_grad) {
            chunk16 old = zero16, gt = zero16, rr;
            if (accum) old = *reinterpret_cast<const chunk16 *>(dst);
            if (gate) gt = glate[it];
#pragma unroll
            for (int j = 0; j < 4; ++j) rr[j] = grad_epilogue_pair(v[j], old[j], gt[j], accum != 0, gate != nullptr);
            *reinterpret_cast<chunk16 *>(dst) = rr;
        } else {
            *reinterpret_cast<chunk16 *>(dst) = v;
        }
    }
}

hipError_t launch_halo(const void *in, const void *wt, const float *bias, void *out, int relu, GradEpi epi,
                       const GatherConv &g, void *pool_out, uint8_t *pool_idx, hipStream_t s)
{
    constexpr int BC = halo_cfg::BC;
    constexpr size_t ring_bytes = (size_t)halo_cfg::ELEMS * 2 + halo_cfg::WS * (size_t)BC * halo_cfg::KS * 2;
    constexpr size_t smem = ring_bytes + BC * sizeof(float);
    static_assert((size_t)256 * (BC + 4) * 2 <= ring_bytes, "epilogue staging fits");
    static_assert((smem + 1279) / 1280 * halo_cfg::BLOCKS_PER_CU <= 128, "blocks per CU (LDS is handed out in 1280-byte granules)");
    auto kfn = k_conv3x3_halo;
    static bool attr_set = false;
    if (!attr_set && smem > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)kfn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int is_grad = (epi.gate != nullptr || epi.accum) ? 1 : 0;
    const unsigned in_bytes = (unsigned)((size_t)g.N * g.Hi * g.Wi * g.Ci * 2);
    const unsigned wt_bytes = (unsigned)((size_t)g.Co * 9 * g.Ci * 2);
    dim3 grid((unsigned)(g.N * (g.Ho / PATCH) * (g.Wo / PATCH) * (g.Co / BC)));
    hipLaunchKernelGGL(kfn, grid, dim3(256), smem, s, (const bf16_t *)in, (const bf16_t *)wt, bias, (bf16_t *)out,
                       (const bf16_t *)epi.gate, epi.accum, relu, is_grad, g.N, g.Hi, g.Wi, g.Ci, g.Co, in_bytes,
                       wt_bytes, (bf16_t *)pool_out, pool_idx);
    return hipGetLastError();
}


// ------------------------------------------------------------------------------------------
// first layer: 8 (padded) input channels
// ------------------------------------------------------------------------------------------
// 3x3 / stride 1 / pad 1 convolution of an input with 8 channels in memory (RGB zero-padded to 8) to
// 64-channel tiles on 16-aligned maps.  There is almost no arithmetic (K = 72): the layer is bound by
// writing its output, so a block is kept small - one 16x16 patch, a 5 KB halo, the whole 64x72 filter
// in registers straight from L2 - and four of them share a CU.  One pixel of the halo is exactly one
// 16-byte MFMA operand chunk: sub-step kk multiplies taps 2kk and 2kk+1 (the 10th tap is a zero filter).
__global__ __launch_bounds__(256, 4) void k_conv3x3_c8(const bf16_t *__restrict__ in, const bf16_t *__restrict__ wt,
                                                       const float *__restrict__ bias, bf16_t *__restrict__ out,
                                                       int relu, int N, int H, int W, int Co, unsigned in_bytes)
{
    constexpr int NW = 4, BC = 64, SROW = BC + 4;
    constexpr unsigned OOB = 0x80000000u;
    extern __shared__ __align__(16) unsigned char smem[];
    const lds_addr_of lds_of(smem);
    uint16_t *sO = reinterpret_cast<uint16_t *>(smem);                        // [256][SROW] (epilogue)
    uint16_t *halo = sO;                                                      // [324 (+60)][8], dead before sO is written
    float *sBias = reinterpret_cast<float *>(sO + 256 * SROW);                // [64]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tiles_c = Co / BC, px_tiles = W / PATCH, py_tiles = H / PATCH;
    const int bid = xcd_remap(blockIdx.x, gridDim.x);
    const int tile_c = bid % tiles_c;
    int t = bid / tiles_c;
    const int X0 = (t % px_tiles) * PATCH;
    t /= px_tiles;
    const int Y0 = (t % py_tiles) * PATCH;
    const int n = t / py_tiles;
    const int co0 = tile_c * BC;

    __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(in), 0, (int)in_bytes, 0x00020000);
    // halo: 324 pixels of 16 bytes = 6 wave-loads (waves 0 and 1 take two, waves 2 and 3 one)
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int q = i * NW + wave;
        if (q < 6) {
            const int hr = q * 64 + lane;
            const int hy = hr / HALO, hx = hr - hy * HALO;
            const int y = Y0 - 1 + hy, x = X0 - 1 + hx;
            const bool ok = hr < HPIX && (unsigned)y < (unsigned)H && (unsigned)x < (unsigned)W;
            dma16(xrsrc, lds_of(halo + q * 512), ok ? (unsigned)((n * H + y) * W + x) * 16u : OOB);
        }
    }
    if (tid < BC) sBias[tid] = bias ? bias[co0 + tid] : 0.0f;

    // the filter, as MFMA operand fragments: lane -> output channel a*32 + (lane & 31), tap 2kk + (lane >> 5)
    const int frow = lane & 31, fhalf = lane >> 5;
    const chunk16 zero16 = {0u, 0u, 0u, 0u};
    chunk16 fw[2][5];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int kk = 0; kk < 5; ++kk) {
            const int tap = 2 * kk + fhalf;
            fw[a][kk] = tap < 9 ? *reinterpret_cast<const chunk16 *>(wt + ((size_t)(co0 + a * 32 + frow) * 9 + tap) * 8) : zero16;
        }

    f32x16_t acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;

    const int py = 4 * wave + (frow >> 4), px = frow & 15;       // patch pixel of B tile 0 (tile 1: py + 2)
    __builtin_amdgcn_s_waitcnt(0x0070);                           // halo, filter and bias: everything has landed
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 5; ++kk) {
        const int tap = 2 * kk + fhalf < 9 ? 2 * kk + fhalf : 8;  // the 10th tap multiplies a zero filter
        const int r = tap / 3, q = tap - r * 3;
        bf16x8_t fb[2];
#pragma unroll
        for (int b = 0; b < 2; ++b)
            fb[b] = as_frag(*reinterpret_cast<const chunk16 *>(halo + ((py + r + 2 * b) * HALO + px + q) * 8));
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b)
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(fw[a][kk]), fb[b], acc[a][b], 0, 0, 0);
    }

    // epilogue: as in the halo kernel (stage [pixel][channel] in LDS, leave as 16-byte rows)
    __syncthreads();                                              // every wave has read its halo pixels
#pragma unroll
    for (int a = 0; a < 2; ++a) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int col = a * 32 + 8 * q + 4 * fhalf;
            const float4 bv = *reinterpret_cast<const float4 *>(sBias + col);
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                const int prow = wave * 64 + b * 32 + frow;
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
    __syncthreads();
#pragma unroll
    for (int it = 0; it < 8; ++it) {
        const int u = tid + it * 256;
        const int pj = u >> 3, c8i = u & 7;
        const size_t p = (size_t)(n * H + Y0 + (pj >> 4)) * W + X0 + (pj & 15);
        const chunk8 lo = *reinterpret_cast<const chunk8 *>(sO + pj * SROW + c8i * 8);
        const chunk8 hi = *reinterpret_cast<const chunk8 *>(sO + pj * SROW + c8i * 8 + 4);
        const chunk16 v = {lo[0], lo[1], hi[0], hi[1]};
        *reinterpret_cast<chunk16 *>(out + p * Co + co0 + c8i * 8) = v;
    }
}

// ------------------------------------------------------------------------------------------
// wgrad with the input halo in LDS
// ------------------------------------------------------------------------------------------
// dw[ko][r][s][c] += sum over pixels of dy[pixel][ko] * x[pixel shifted by tap (r,s)][c] for 3x3 /
// stride 1 / pad 1 on 16-aligned maps.  A block owns 64 output channels x 64 input channels x ALL 9
// taps (a 64 x 576 fp32 tile, 144 accumulator registers per lane) and walks over units of 8x16
// pixels: the unit's dy rows and the 10x18 halo of x land in LDS once (buffer_load ... lds, two
// stages) and the nine taps read shifted views of the same halo through the transposing LDS read,
// so x is fetched 1.4 times instead of 9.  Units are split over blockIdx.y; partial tiles are
// reduced by k_wg_halo_reduce in a fixed order.
constexpr int UH = 8, UW = 16, UPIX = UH * UW;                 // unit of 8 x 16 pixels
constexpr int WH_ROWS = UH + 2, WH_COLS = UW + 2, WH_PIX = WH_ROWS * WH_COLS;      // 10 x 18 halo = 180 pixels
constexpr int WG_DY_ELEMS = UPIX * 64;                         // 16 KB
constexpr int WG_HALO_ELEMS = WH_PIX * 64 + 256;               // 1440 slots + 32 slots the last wave-load overruns
constexpr int WG_STAGE_ELEMS = WG_DY_ELEMS + WG_HALO_ELEMS;
constexpr int WG_HL = 6, WG_DL = 4;                            // wave-loads per wave: halo (24 >= 22.5), dy (16)

__global__ __launch_bounds__(256, 2) void k_wgrad3x3_halo(const bf16_t *__restrict__ x, const bf16_t *__restrict__ dy,
                                                          float *__restrict__ part, int N, int H, int W, int C,
                                                          int K, int units_per_split, unsigned x_bytes,
                                                          unsigned dy_bytes, int with_bias)
{
    constexpr unsigned OOB = 0x80000000u;
    constexpr int NW = 4;
    extern __shared__ __align__(16) unsigned char smem[];
    const lds_addr_of lds_of(smem);
    uint16_t *stage0 = reinterpret_cast<uint16_t *>(smem);
    uint16_t *dump = stage0 + 2 * WG_STAGE_ELEMS;              // 64 slots for the one all-out-of-range wave-load

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wk = wave & 1, wn = wave >> 1;                   // 32 output channels x 9 column tiles per wave
    const int cslices = C / 64;
    // The (output-channel, input-channel) tiles of one split read the same dy rows and x halos: number the
    // blocks so that they run on the same XCD (one L2) at the same time - consecutive block ids go round the
    // eight XCDs, so each XCD is given a contiguous range of (split, tile) positions
    const int tiles = (int)gridDim.x;
    const int pos = xcd_remap((int)(blockIdx.y * gridDim.x + blockIdx.x), tiles * (int)gridDim.y);
    const int tile = pos % tiles, split = pos / tiles;
    const int cs = tile % cslices, kt = tile / cslices;
    const int ko0 = kt * 64, ci0 = cs * 64;
    const int ux = W / UW, uy = H / UH, upi = ux * uy;
    const int U = N * upi;
    const int u0 = split * units_per_split;
    const int u1 = u0 + units_per_split < U ? u0 + units_per_split : U;

    __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(x), 0, (int)x_bytes, 0x00020000);
    __amdgpu_buffer_rsrc_t grsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(dy), 0, (int)dy_bytes, 0x00020000);

    // halo slots of this lane (fixed relative to the unit origin)
    int hdy[WG_HL], hdx[WG_HL];
    unsigned hco[WG_HL];
#pragma unroll
    for (int i = 0; i < WG_HL; ++i) {
        const int slot = (i * NW + wave) * 64 + lane;
        const int hr = slot >> 3, cq = slot & 7;
        const int c = ((((cq >> 1) ^ wg_swz<64>(hr)) << 1) | (cq & 1));
        const int hy = hr / WH_COLS, hx = hr - hy * WH_COLS;
        hdy[i] = hr < WH_PIX ? hy - 1 : -(1 << 20);
        hdx[i] = hx - 1;
        hco[i] = (unsigned)(ci0 + c * 8) * 2u;
    }
    unsigned dco[WG_DL];
    int ddy[WG_DL], ddx[WG_DL];
#pragma unroll
    for (int i = 0; i < WG_DL; ++i) {
        const int slot = (i * NW + wave) * 64 + lane;
        const int px = slot >> 3, cq = slot & 7;
        const int c = ((((cq >> 1) ^ wg_swz<64>(px)) << 1) | (cq & 1));
        ddy[i] = px >> 4;
        ddx[i] = px & 15;
        dco[i] = (unsigned)(ko0 + c * 8) * 2u;
    }
    auto issue_unit = [&](int u, int st) {
        uint16_t *sd = stage0 + st * WG_STAGE_ELEMS, *sh = sd + WG_DY_ELEMS;
        const bool live = u < u1;
        const int n = u / upi, rem = u - n * upi;
        const int Y0 = (rem / ux) * UH, X0 = (rem % ux) * UW;
#pragma unroll
        for (int i = 0; i < WG_DL; ++i) {
            unsigned vo = live ? (unsigned)(((n * H + Y0 + ddy[i]) * W + X0 + ddx[i]) * K) * 2u + dco[i] : OOB;
            dma16(grsrc, lds_of(sd + (i * NW + wave) * 512), vo);
        }
#pragma unroll
        for (int i = 0; i < WG_HL; ++i) {
            const int y = Y0 + hdy[i], xx = X0 + hdx[i];
            const bool ok = live && (unsigned)y < (unsigned)H && (unsigned)xx < (unsigned)W;
            unsigned vo = ok ? (unsigned)(((n * H + y) * W + xx) * C) * 2u + hco[i] : OOB;
            const int q = i * NW + wave;                             // wave-load 23 lies wholly past the halo
            uint16_t *dst = q * 64 < WH_PIX * 8 ? sh + q * 512 : dump;
            dma16(xrsrc, lds_of(dst), vo);
        }
    };

    f32x16_t acc[9];
#pragma unroll
    for (int b = 0; b < 9; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[b][v] = 0.0f;

    // bias gradient = column sums of dy: the waves that hold the dy fragments of input-channel slice 0
    // add up their fragment values on the side (lane -> output channel, 8 pixels per step)
    const bool do_bias = with_bias && cs == 0 && wn == 0;
    float bsum = 0.0f;

    // Fragment addresses (element offsets into a stage).  A fragment's swizzle depends on bit 1 of
    // its pixel row, which moving down two halo rows (36 pixels) or one dy row (16 pixels) leaves
    // alone, so one offset per column tile and row parity is enough; the row itself becomes the
    // immediate offset of the read.
    auto frag_off = [&](int ch0, int k0) {
        const int blk = lane >> 4, sl = lane & 15;
        const int row = k0 + 8 * (blk >> 1) + (sl >> 2);
        const int col = ch0 + 16 * (blk & 1) + 4 * (sl & 3);
        const int chunk = col >> 3;
        const int sw = (((chunk >> 1) ^ wg_swz<64>(row)) << 1) | (chunk & 1);
        return row * 64 + (sw << 3) + (col & 7);
    };
    auto frag_at = [&](const uint16_t *p) {
        typedef __attribute__((address_space(3))) s16x4_t lds_v4;
        typedef short s16x8_t __attribute__((ext_vector_type(8)));
        s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4 *)(p));
        s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4 *)(p + 4 * 64));
        return __builtin_bit_cast(bf16x8_t, (s16x8_t)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    const int offA = frag_off(wk * 32, 0);
    int offB[9][2];
#pragma unroll
    for (int b = 0; b < 9; ++b) {
        const int ct = wn * 9 + b, tap = ct >> 1;
        const int r = tap / 3, q = tap - r * 3;
        offB[b][0] = WG_DY_ELEMS + frag_off((ct & 1) * 32, r * WH_COLS + q);
        offB[b][1] = WG_DY_ELEMS + frag_off((ct & 1) * 32, (r + 1) * WH_COLS + q);
    }

    // Main loop.  One unit = 8 pixel rows x 9 column tiles = 72 MFMAs per wave, fully unrolled; the
    // x fragment of MFMA j+2 and the dy fragment of the next row are requested before MFMA j is
    // issued (sched_barrier keeps that order), so the LDS latency hides behind two MFMAs.
    issue_unit(u0, 0);
    WAIT_LGKMCNT(0);           // no scalar load pending at loop entry (else every LDS wait becomes a full drain)
    for (int u = u0; u < u1; ++u) {
        const int st = (u - u0) & 1;
        WAIT_VMCNT(0);
        __builtin_amdgcn_s_barrier();
        issue_unit(u + 1, st ^ 1);
        const uint16_t *sd = stage0 + st * WG_STAGE_ELEMS;
        auto ld_b = [&](int j) {                                   // x fragment of MFMA j = (row j/9, tile j%9)
            const int y = j / 9, bb = j % 9;
            return frag_at(sd + offB[bb][y & 1] + (y & ~1) * WH_COLS * 64);
        };
        bf16x8_t fa_cur = frag_at(sd + offA), fa_nxt = fa_cur;
        bf16x8_t fbq[3];
        fbq[0] = ld_b(0);
        fbq[1] = ld_b(1);
#pragma unroll
        for (int j = 0; j < UH * 9; ++j) {
            const int y = j / 9, bb = j % 9;
            if (j + 2 < UH * 9) fbq[(j + 2) % 3] = ld_b(j + 2);
            if (bb == 4 && y + 1 < UH) fa_nxt = frag_at(sd + offA + (y + 1) * 16 * 64);
            __builtin_amdgcn_sched_barrier(0);
            if (bb == 0 && do_bias) bsum = frag_sum(fa_cur, bsum);
            acc[bb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa_cur, fbq[j % 3], acc[bb], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if (bb == 8) fa_cur = fa_nxt;
        }
    }
    WAIT_VMCNT(0);

    // partial[split][ko][tap][c] followed by the bias partial [split][ko]: a wave writes 32 consecutive
    // c (128 bytes) per row
    const size_t total_w = (size_t)K * 9 * C;
    float *dst = part + (size_t)split * (total_w + (with_bias ? K : 0));
    const int col = lane & 31, half = lane >> 5;
    if (do_bias) {
        bsum += __shfl_xor(bsum, 32, 64);
        if (half == 0) dst[total_w + ko0 + wk * 32 + col] = bsum;
    }
#pragma unroll
    for (int b = 0; b < 9; ++b) {
        const int ct = wn * 9 + b, tap = ct >> 1;
        const int c = ci0 + (ct & 1) * 32 + col;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int ko = ko0 + wk * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
            dst[((size_t)ko * 9 + tap) * C + c] = acc[b][v];
        }
    }
}

// dw[i] += sum_k part[k][i] for i < total_w, db[i - total_w] += ... for the bias tail (total_w and
// total are multiples of 4); split lanes are combined through LDS in a fixed order.
__global__ void k_wg_halo_reduce(const float *__restrict__ part, float *dw, float *db, size_t total_w, size_t total,
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

// ------------------------------------------------------------------------------------------
// wgrad of the first layer: 8 (padded) input channels
// ------------------------------------------------------------------------------------------
// dw[ko][tap][c] for an input with 8 channels in memory: a 64 x 72 tile per block, next to no arithmetic,
// so the kernel only has to stream dy once.  Units of 8x16 pixels as above (dy rows and the 10x18 halo
// of x by buffer_load ... lds, two stages); the four waves split the unit's pixels (32 each) and every
// wave keeps the whole 64 x 96 tile (72 columns used), the waves' tiles being added through LDS once
// at the end.  dy fragments come from the transposing LDS read; an x fragment - 8 consecutive pixels
// of one (tap, channel) column - is gathered with eight 2-byte reads from the plain [pixel][8] halo.
constexpr int C8W_HALO_ELEMS = 192 * 8;                        // 180 halo pixels, three wave-loads
constexpr int C8W_STAGE_ELEMS = WG_DY_ELEMS + C8W_HALO_ELEMS;
constexpr int C8W_LD = 96 + 1;                                 // row of the end-of-block reduction tile

__global__ __launch_bounds__(256, 2) void k_wgrad3x3_c8(const bf16_t *__restrict__ x, const bf16_t *__restrict__ dy,
                                                        float *__restrict__ part, int N, int H, int W, int K,
                                                        int units_per_split, unsigned x_bytes, unsigned dy_bytes,
                                                        int with_bias)
{
    constexpr unsigned OOB = 0x80000000u;
    constexpr int NW = 4;
    extern __shared__ __align__(16) unsigned char smem[];
    const lds_addr_of lds_of(smem);
    uint16_t *stage0 = reinterpret_cast<uint16_t *>(smem);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ko0 = blockIdx.x * 64;
    const int ux = W / UW, uy = H / UH, upi = ux * uy;
    const int U = N * upi;
    const int u0 = blockIdx.y * units_per_split;
    const int u1 = u0 + units_per_split < U ? u0 + units_per_split : U;

    __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(x), 0, (int)x_bytes, 0x00020000);
    __amdgpu_buffer_rsrc_t grsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(dy), 0, (int)dy_bytes, 0x00020000);

    unsigned dco[WG_DL];
    int ddy[WG_DL], ddx[WG_DL];
#pragma unroll
    for (int i = 0; i < WG_DL; ++i) {
        const int slot = (i * NW + wave) * 64 + lane;
        const int px = slot >> 3, cq = slot & 7;
        const int c = ((((cq >> 1) ^ wg_swz<64>(px)) << 1) | (cq & 1));
        ddy[i] = px >> 4;
        ddx[i] = px & 15;
        dco[i] = (unsigned)(ko0 + c * 8) * 2u;
    }
    const int hr = wave * 64 + lane;                           // halo pixel of this lane (waves 0..2)
    const int hdy = hr / WH_COLS - 1, hdx = hr % WH_COLS - 1;
    auto issue_unit = [&](int u, int st) {
        uint16_t *sd = stage0 + st * C8W_STAGE_ELEMS, *sh = sd + WG_DY_ELEMS;
        const bool live = u < u1;
        const int n = u / upi, rem = u - n * upi;
        const int Y0 = (rem / ux) * UH, X0 = (rem % ux) * UW;
#pragma unroll
        for (int i = 0; i < WG_DL; ++i) {
            unsigned vo = live ? (unsigned)(((n * H + Y0 + ddy[i]) * W + X0 + ddx[i]) * K) * 2u + dco[i] : OOB;
            dma16(grsrc, lds_of(sd + (i * NW + wave) * 512), vo);
        }
        if (wave < 3) {
            const int y = Y0 + hdy, xx = X0 + hdx;
            const bool ok = live && hr < WH_PIX && (unsigned)y < (unsigned)H && (unsigned)xx < (unsigned)W;
            dma16(xrsrc, lds_of(sh + wave * 512), ok ? (unsigned)((n * H + y) * W + xx) * 16u : OOB);
        }
    };

    f32x16_t acc[2][3];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 3; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;
    float bsum[2] = {0.0f, 0.0f};

    // x fragment addressing: column n = b*32 + (lane & 31) is (tap, channel) = (n / 8, n % 8); the 8 pixels
    // of a fragment lie in one row of the unit, so they are 8 consecutive halo pixels
    const int frow = lane & 31, fhalf = lane >> 5;
    int xoff[3];                                               // element offset of pixel 0 of the unit under the lane's tap
    bool xin[3];
#pragma unroll
    for (int b = 0; b < 3; ++b) {
        const int nn = b * 32 + frow, tap = nn >> 3, c = nn & 7;
        xin[b] = nn < 72;
        xoff[b] = xin[b] ? ((tap / 3) * WH_COLS + tap % 3) * 8 + c : 0;
    }

    issue_unit(u0, 0);
    WAIT_LGKMCNT(0);
    for (int u = u0; u < u1; ++u) {
        const int st = (u - u0) & 1;
        WAIT_VMCNT(0);
        __builtin_amdgcn_s_barrier();
        issue_unit(u + 1, st ^ 1);
        const uint16_t *sd = stage0 + st * C8W_STAGE_ELEMS, *sh = sd + WG_DY_ELEMS;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const int k0 = wave * 32 + ks * 16;                // first pixel of this K-step (this wave's 32 pixels)
            const int p = k0 + 8 * fhalf;                      // first of the lane's 8 pixels: row p / 16, column p % 16
            const int hbase = ((p >> 4) * WH_COLS + (p & 15)) * 8;
            bf16x8_t fa[2], fb[3];
#pragma unroll
            for (int a = 0; a < 2; ++a) fa[a] = tr_frag<64>(sd, a * 32, k0, lane);
#pragma unroll
            for (int b = 0; b < 3; ++b) {
                chunk16 v = {0u, 0u, 0u, 0u};
                if (xin[b]) {
                    const uint16_t *q = sh + hbase + xoff[b];
#pragma unroll
                    for (int j = 0; j < 4; ++j) v[j] = (uint32_t)q[16 * j] | ((uint32_t)q[16 * j + 8] << 16);
                }
                fb[b] = as_frag(v);
            }
            if (with_bias) {
#pragma unroll
                for (int a = 0; a < 2; ++a) bsum[a] = frag_sum(fa[a], bsum[a]);
            }
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 3; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
        }
    }
    WAIT_VMCNT(0);
    __syncthreads();

    // add the four waves' tiles in wave order through LDS: red[ko 64][n 96], then the bias sums
    float *red = reinterpret_cast<float *>(smem);
    float *bred = red + 64 * C8W_LD;                           // [4 waves][64]
    for (int w = 0; w < NW; ++w) {
        if (wave == w) {
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 3; ++b)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        float *q = red + (a * 32 + 8 * (v >> 2) + 4 * fhalf + (v & 3)) * C8W_LD + b * 32 + frow;
                        *q = w == 0 ? acc[a][b][v] : *q + acc[a][b][v];
                    }
        }
        __syncthreads();
    }
    if (with_bias) {
#pragma unroll
        for (int a = 0; a < 2; ++a) {
            const float t = bsum[a] + __shfl_xor(bsum[a], 32, 64);
            if (fhalf == 0) bred[wave * 64 + a * 32 + frow] = t;
        }
        __syncthreads();
    }
    const size_t total_w = (size_t)K * 72;
    float *dst = part + (size_t)blockIdx.y * (total_w + (with_bias ? K : 0));
    for (int i = tid; i < 64 * 72; i += 256) {
        const int ko = i / 72, nn = i - ko * 72;
        dst[(size_t)(ko0 + ko) * 72 + nn] = red[ko * C8W_LD + nn];
    }
    if (with_bias && tid < 64) dst[total_w + ko0 + tid] = (bred[tid] + bred[64 + tid]) + (bred[128 + tid] + bred[192 + tid]);
}

struct WgHaloPlan {
    int tiles, splits, units_per_split;
};

WgHaloPlan wg_halo_plan(const ConvShape &c)
{
    WgHaloPlan p;
    p.tiles = (c.K / 64) * (c.C / 64);
    const int U = c.N * (c.H / UH) * (c.W / UW);
    // One block per compute unit: every block writes a full fp32 copy of its tile, so the traffic of the partial
    // sums grows with the block count (at 512 blocks it was a ninth of the first VGG stage's HBM bytes), and a
    // second block per unit made the kernel only 5 % faster on its own; beside kernels of other streams fewer,
    // longer blocks are the better neighbour.
    int want = (256 + p.tiles - 1) / p.tiles;
    if (want > U) want = U;
    if (want < 1) want = 1;
    p.units_per_split = (U + want - 1) / want;
    p.splits = (U + p.units_per_split - 1) / p.units_per_split;
    return p;
}

}  // namespace

bool conv3x3_halo_supported(const GatherConv &g)
{
    return g.R == 3 && g.S == 3 && g.s_out == 1 && g.s_in == 1 && g.pad_h == 1 && g.pad_w == 1 && g.Hi == g.Ho &&
           g.Wi == g.Wo && g.Ho % PATCH == 0 && g.Wo % PATCH == 0 && g.Ci % 64 == 0 && g.Co % 64 == 0 &&
           (long long)g.N * g.Hi * g.Wi * g.Ci * 2 < (1ll << 31) && (long long)g.Co * 9 * g.Ci * 2 < (1ll << 31) &&
           (long long)g.N * g.Ho * g.Wo * g.Co < (1ll << 40);
}

hipError_t conv3x3_halo_mfma(const void *in, const void *wt, const float *bias, void *out, int relu,
                             GradEpi epi, const GatherConv &g, hipStream_t s)
{
    if (!conv3x3_halo_supported(g)) return hipErrorInvalidValue;
    return launch_halo(in, wt, bias, out, relu, epi, g, nullptr, nullptr, s);
}

bool conv3x3_c8_supported(const GatherConv &g)
{
    return g.R == 3 && g.S == 3 && g.s_out == 1 && g.s_in == 1 && g.pad_h == 1 && g.pad_w == 1 && g.Hi == g.Ho &&
           g.Wi == g.Wo && g.Ho % PATCH == 0 && g.Wo % PATCH == 0 && g.Ci == 8 && g.Co % 64 == 0 &&
           (long long)g.N * g.Hi * g.Wi * 16 < (1ll << 31) && (long long)g.N * g.Ho * g.Wo * g.Co < (1ll << 40);
}

hipError_t conv3x3_c8_mfma(const void *in, const void *wt, const float *bias, void *out, int relu,
                           const GatherConv &g, hipStream_t s)
{
    if (!conv3x3_c8_supported(g)) return hipErrorInvalidValue;
    constexpr size_t smem = (size_t)256 * 68 * 2 + 64 * sizeof(float);
    static_assert(smem <= 40 * 1024, "four blocks per CU");
    const unsigned in_bytes = (unsigned)((size_t)g.N * g.Hi * g.Wi * 16);
    dim3 grid((unsigned)(g.N * (g.Ho / PATCH) * (g.Wo / PATCH) * (g.Co / 64)));
    hipLaunchKernelGGL(k_conv3x3_c8, grid, dim3(256), smem, s, (const bf16_t *)in, (const bf16_t *)wt, bias,
                       (bf16_t *)out, relu, g.N, g.Hi, g.Wi, g.Co, in_bytes);
    return hipGetLastError();
}

hipError_t conv3x3_halo_pool_mfma(const void *in, const void *wt, const float *bias, int relu, void *pool_out,
                                  uint8_t *pool_idx, const GatherConv &g, hipStream_t s)
{
    if (!conv3x3_halo_supported(g) || !pool_out || !pool_idx || ((uintptr_t)pool_idx & 7)) return hipErrorInvalidValue;
    GradEpi none{nullptr, 0};
    return launch_halo(in, wt, bias, nullptr, relu, none, g, pool_out, pool_idx, s);
}

}  // namespace bapipe

namespace bapipe {

bool wgrad3x3_c8_supported(const ConvShape &c)
{
    return c.R == 3 && c.S == 3 && c.stride == 1 && c.pad == 1 && c.H == c.P && c.W == c.Q && c.H % UH == 0 &&
           c.W % UW == 0 && c.C == 8 && c.K % 64 == 0 && (long long)c.N * c.H * c.W * 16 < (1ll << 31) &&
           (long long)c.N * c.H * c.W * c.K * 2 < (1ll << 31);
}

static WgHaloPlan wg_c8_plan(const ConvShape &c)
{
    WgHaloPlan p;
    p.tiles = c.K / 64;
    const int U = c.N * (c.H / UH) * (c.W / UW);
    // One block per compute unit: every block writes a full fp32 copy of its tile, so the traffic of the partial
    // sums grows with the block count (at 512 blocks it was a ninth of the first VGG stage's HBM bytes), and a
    // second block per unit made the kernel only 5 % faster on its own; beside kernels of other streams fewer,
    // longer blocks are the better neighbour.
    int want = (256 + p.tiles - 1) / p.tiles;
    if (want > U) want = U;
    if (want < 1) want = 1;
    p.units_per_split = (U + want - 1) / want;
    p.splits = (U + p.units_per_split - 1) / p.units_per_split;
    return p;
}

size_t wgrad3x3_c8_workspace(const ConvShape &c)
{
    return (size_t)wg_c8_plan(c).splits * ((size_t)c.K * 72 + c.K) * sizeof(float);
}

hipError_t wgrad3x3_c8_mfma(const void *x, const void *dy, float *dw, float *db, void *workspace, const ConvShape &c,
                            hipStream_t s)
{
    if (!wgrad3x3_c8_supported(c)) return hipErrorInvalidValue;
    const WgHaloPlan p = wg_c8_plan(c);
    constexpr size_t stages = (size_t)2 * C8W_STAGE_ELEMS * 2, redb = (size_t)(64 * C8W_LD + 256) * sizeof(float);
    constexpr size_t smem = stages > redb ? stages : redb;
    static_assert(smem <= 64 * 1024, "no attribute needed, two blocks per CU");
    const unsigned x_bytes = (unsigned)((size_t)c.N * c.H * c.W * 16);
    const unsigned dy_bytes = (unsigned)((size_t)c.N * c.H * c.W * c.K * 2);
    float *part = (float *)workspace;
    hipLaunchKernelGGL(k_wgrad3x3_c8, dim3((unsigned)p.tiles, (unsigned)p.splits), dim3(256), smem, s, (const bf16_t *)x,
                       (const bf16_t *)dy, part, c.N, c.H, c.W, c.K, p.units_per_split, x_bytes, dy_bytes, db ? 1 : 0);
    const size_t total_w = (size_t)c.K * 72, total = total_w + (db ? c.K : 0);
    hipLaunchKernelGGL(k_wg_halo_reduce, dim3((unsigned)((total / 4 + 63) / 64)), dim3(256), 0, s, part, dw, db,
                       total_w, total, p.splits);
    return hipGetLastError();
}

bool wgrad3x3_halo_supported(const ConvShape &c)
{
    return c.R == 3 && c.S == 3 && c.stride == 1 && c.pad == 1 && c.H == c.P && c.W == c.Q && c.H % UH == 0 &&
           c.W % UW == 0 && c.C % 64 == 0 && c.K % 64 == 0 &&
           (long long)c.N * c.H * c.W * c.C * 2 < (1ll << 31) && (long long)c.N * c.H * c.W * c.K * 2 < (1ll << 31);
}

size_t wgrad3x3_halo_workspace(const ConvShape &c)
{
    return (size_t)wg_halo_plan(c).splits * ((size_t)c.K * 9 * c.C + c.K) * sizeof(float);
}

hipError_t wgrad3x3_halo_mfma(const void *x, const void *dy, float *dw, float *db, void *workspace,
                              const ConvShape &c, hipStream_t s)
{
    if (!wgrad3x3_halo_supported(c)) return hipErrorInvalidValue;
    const WgHaloPlan p = wg_halo_plan(c);
    constexpr size_t smem = (size_t)(2 * WG_STAGE_ELEMS + 512) * 2;
    static_assert(smem <= 80 * 1024, "two blocks per CU");
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)k_wgrad3x3_halo, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const unsigned x_bytes = (unsigned)((size_t)c.N * c.H * c.W * c.C * 2);
    const unsigned dy_bytes = (unsigned)((size_t)c.N * c.H * c.W * c.K * 2);
    float *part = (float *)workspace;
    hipLaunchKernelGGL(k_wgrad3x3_halo, dim3((unsigned)p.tiles, (unsigned)p.splits), dim3(256), smem, s,
                       (const bf16_t *)x, (const bf16_t *)dy, part, c.N, c.H, c.W, c.C, c.K, p.units_per_split,
                       x_bytes, dy_bytes, db ? 1 : 0);
    const size_t total_w = (size_t)c.K * 9 * c.C, total = total_w + (db ? c.K : 0);
    hipLaunchKernelGGL(k_wg_halo_reduce, dim3((unsigned)((total / 4 + 63) / 64)), dim3(256), 0, s, part, dw, db,
                       total_w, total, p.splits);
    return hipGetLastError();
}

}  // namespace bapipe
