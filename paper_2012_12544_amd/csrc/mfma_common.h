// Pieces shared by the MFMA kernels (gfx950): operand fragment types, the vmcnt-only wait, the
// XCD-aware block order and the transposing-read fragment loader of the weight-gradient kernels.
#pragma once
#include "dev_common.h"

namespace bapipe {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef uint32_t chunk16 __attribute__((ext_vector_type(4)));   // 8 bf16, one 16-byte access
typedef uint32_t chunk8 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) void lds_void_t;

// s_waitcnt with only the vector-memory counter set: wait until at most n loads are in flight
#define WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14))
// ... with only the LDS / scalar-memory counter set
#define WAIT_LGKMCNT(n) __builtin_amdgcn_s_waitcnt(0xC07F | ((n) << 8))

// One wave-wide 16-byte-per-lane load HBM/L2 -> LDS (buffer_load_dwordx4 ... lds): lane l's chunk lands
// at LDS byte address lds_addr + 16*l (wave-uniform); a lane whose voffset is outside the buffer gets
// zeros.  Written as inline assembly on purpose: when the compiler knows of an LDS-DMA in flight it
// puts s_waitcnt vmcnt(0) in front of every transposing LDS read (it cannot tell which bytes the DMA
// writes), which would drain the prefetch ring once per K-step.  Completion is tracked by hand with
// WAIT_VMCNT in every kernel that uses this; loads the compiler does track only wait longer for it.
// No "memory" clobber: the s_barrier / s_waitcnt builtins around it already pin the LDS accesses,
// and with one the LDS reads could no longer be scheduled around the issue slots.
__device__ __forceinline__ void dma16(__amdgpu_buffer_rsrc_t rsrc, unsigned lds_addr, unsigned voffset)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" ::"s"(lds_addr), "v"(voffset), "s"(rsrc));
}

// LDS byte address of a pointer into the kernel's dynamic shared memory, for dma16: base address taken
// once, the rest is integer arithmetic (a generic pointer cast per load would cost a null check each)
struct lds_addr_of {
    const unsigned char *base;
    unsigned addr0;
    __device__ __forceinline__ explicit lds_addr_of(const unsigned char *smem)
        : base(smem), addr0((unsigned)(uintptr_t)(lds_void_t *)smem) {}
    __device__ __forceinline__ unsigned operator()(const void *p) const
    {
        return __builtin_amdgcn_readfirstlane(addr0 + (unsigned)((const unsigned char *)p - base));
    }
};

__device__ __forceinline__ bf16x8_t as_frag(chunk16 c) { return __builtin_bit_cast(bf16x8_t, c); }

// XCD-aware block order: hardware deals consecutive block ids round-robin to the 8 XCDs
// (each with its own L2).  Re-number so that every XCD walks one contiguous range of tiles
// and the blocks that share an input tile run on the same L2.
__device__ __forceinline__ int xcd_remap(int id, int nb)
{
    const int x = id & 7, q = nb >> 3, rem = nb & 7;
    return x * q + (x < rem ? x : rem) + (id >> 3);
}

// acc + the 8 bf16 values of an MFMA operand fragment (v_dot2c_f32_bf16 against a pair of ones)
__device__ __forceinline__ float frag_sum(bf16x8_t f, float acc)
{
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    const bf16x2_t ones = __builtin_bit_cast(bf16x2_t, 0x3F803F80u);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(f, f, 0, 1), ones, acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(f, f, 2, 3), ones, acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(f, f, 4, 5), ones, acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(f, f, 6, 7), ones, acc, false);
    return acc;
}

// LDS tile [pixels][CH channels], rows unpadded (they are filled by buffer_load ... lds, whose
// lanes land in consecutive 16-byte slots).  One 16-lane group of a transposing read touches 4
// consecutive pixel rows x 32 bytes; the 32-byte pair index inside a row is XORed with a function of
// the row so that the 32 lanes served together hit 8 different 32-byte bank groups.
template <int CH> __device__ __forceinline__ int wg_swz(int row)
{
    constexpr int PPR = CH / 16;                      // 32-byte pairs per row
    constexpr int RPS = PPR >= 8 ? 1 : 8 / PPR;       // rows per 256-byte bank sweep
    return (2 * ((row / RPS) & 3)) & (PPR - 1);
}

// fragment for v_mfma_f32_32x32x16_bf16 out of a [pixel][channel] LDS tile:
// lane -> channel ch0 + (lane & 31), pixels k0 + 8*(lane >> 5) .. +7  (two transposing reads)
template <int CH>
__device__ __forceinline__ bf16x8_t tr_frag(const uint16_t *tile, int ch0, int k0, int lane)
{
    const int blk = lane >> 4, sl = lane & 15;
    const int row = k0 + 8 * (blk >> 1) + (sl >> 2);
    const int col = ch0 + 16 * (blk & 1) + 4 * (sl & 3);
    const int chunk = col >> 3;
    const int sw = (((chunk >> 1) ^ wg_swz<CH>(row)) << 1) | (chunk & 1);
    const uint16_t *p = tile + row * CH + (sw << 3) + (col & 7);
    typedef __attribute__((address_space(3))) s16x4_t lds_v4;
    s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4 *)(p));
    s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4 *)(p + 4 * CH));     // rows +4: same swizzle
    typedef short s16x8_t __attribute__((ext_vector_type(8)));
    s16x8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8_t, both);
}

}  // namespace bapipe
