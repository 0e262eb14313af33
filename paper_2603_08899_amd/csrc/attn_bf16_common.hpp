// Shared pieces of the bf16 attention kernels for gfx950 (head dimension 128): operand vector types, the LDS layout,
// direct-to-LDS load helpers with hand-tracked completion, and the per-tile visibility word.  Included by the
// translation units that hold the kernels; everything here has internal linkage.
#pragma once

#include "tv_internal.hpp"

namespace tv {

namespace {

// memory is reinterpreted between these vector types (LDS <-> MFMA operands <-> global)
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8), may_alias));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4), may_alias));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4), may_alias));

constexpr int kD = 128;
constexpr int kQRows = 64;                 // packed query rows per row block (unit of the workspace layout)
constexpr int kTK = 32;                    // keys per tile
constexpr int kRowBytes = 256;             // one K or V row of one head in LDS
constexpr int kTileBytes = kTK * kRowBytes;          // 8192: one K tile or one V tile
constexpr int kStageBytes = 2 * kTileBytes;          // K then V
constexpr int kRingBytes = 128 * 1024;               // all stages of all streams; later the merge buffer
constexpr int kWgRows = 256;                         // rows x streams held by the waves of a workgroup
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kTau = 8.f;                // the running max is only raised when it lags by more than 2^kTau

struct Bf16Smem {
    unsigned char big[kRingBytes];         // K/V stage ring, later the merge buffer [256 rows][32 float4]
    float ml[kWgRows][2];                  // (max, sum) of every wave's rows
    int parent[kMaxRows];
    int kind[kMaxRows];                    // low byte = TV_KIND_* (a one-byte direct-to-LDS load fills one dword per row)
    unsigned long long bits[kMaxRows][2];  // ancestor mask of every row (only filled where masked tiles occur)
    int prep_status[kWave];                // verdict of a prepared tree (entry 0; a direct-to-LDS load fills all)
    int flag;
};
// 64-row workgroups stage their query block behind the struct, in an area of its own: the whole stage ring then
// takes K/V tiles from the first instruction on (160 KB of LDS hold 128 KB of ring, 16 KB of Q and the rest).
constexpr int kQAreaOffset = (sizeof(Bf16Smem) + 1023) / 1024 * 1024;
constexpr int kQAreaBytes = kQRows * kRowBytes;
template <int RB> constexpr int smem_bytes() { return RB == 1 ? kQAreaOffset + kQAreaBytes : (int)sizeof(Bf16Smem); }

__device__ __forceinline__ float cross_half_max(float x) {
    // permlane32_swap(a, b) returns {[a.lo, b.lo], [a.hi, b.hi]}: with a = b = x both halves see both values
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float cross_half_sum(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// s_waitcnt vmcnt(n) only (gfx9 encoding: vmcnt = bits [3:0] and [15:14], expcnt [6:4], lgkmcnt [11:8])
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | (((N >> 4) & 3) << 14));
}

// One direct-to-LDS load: every lane fetches 16 bytes from sbase + voff (sbase wave-uniform) and the
// 64 x 16 bytes land contiguously at LDS byte address lds_addr (wave-uniform), lane l at lds_addr + 16*l.
// Written as inline assembly on purpose: the loads stay invisible to the compiler's wait-count
// insertion, which would otherwise put a conservative vmcnt(0) in front of LDS reads and so wait for
// the tiles that were just requested.  Completion is tracked by hand with wait_vmcnt (these loads
// retire in order on the vector-memory counter).
__device__ __forceinline__ void dma16(unsigned lds_addr, unsigned long long sbase, unsigned voff) {
    // (the scalar operands are pinned to SGPRs: an "s" constraint alone does not stop the compiler from
    //  handing over a vector register when it has lost track of a value's uniformity)
    const unsigned m = __builtin_amdgcn_readfirstlane(lds_addr);
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)sbase);
    const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(sbase >> 32));
    const unsigned long long sb = ((unsigned long long)hi << 32) | lo;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(m), "v"(voff), "s"(sb) : "memory", "m0");
}
// The same with 4 bytes (or one zero-extended byte) per lane: lane l lands at lds_addr + 4*l.
__device__ __forceinline__ void dma4(unsigned lds_addr, unsigned long long sbase, unsigned voff) {
    const unsigned m = __builtin_amdgcn_readfirstlane(lds_addr);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
                 :: "s"(m), "v"(voff), "s"(sbase) : "memory", "m0");
}
__device__ __forceinline__ void dma1(unsigned lds_addr, unsigned long long sbase, unsigned voff) {
    const unsigned m = __builtin_amdgcn_readfirstlane(lds_addr);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_ubyte %1, %2"
                 :: "s"(m), "v"(voff), "s"(sbase) : "memory", "m0");
}
// A wave-uniform pointer as a scalar value the assembler operand above accepts (pins it to SGPRs even when
// the compiler cannot prove uniformity).
__device__ __forceinline__ unsigned long long scalar_base(const void* p) {
    const unsigned long long v = (unsigned long long)(uintptr_t)p;
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v);
    const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
    return ((unsigned long long)hi << 32) | lo;
}
__device__ __forceinline__ unsigned lds_address(const void* p) {
    return (unsigned)(uintptr_t)(const void __attribute__((address_space(3)))*)p;
}

// Visibility of the 32 keys of the tile starting at k0 for one query row (bit kk = key k0+kk).
__device__ __forceinline__ unsigned tile_visibility(int k0, int P, int soft_len, bool is_con,
                                                    unsigned long long b0, unsigned long long b1) {
    // cached rows: [soft_len, P) for draft nodes, [0, P) for contemplate rows
    const int lo = is_con ? 0 : max(0, soft_len - k0);
    const int hi = min(32, P - k0);
    unsigned pm = 0;
    if (hi > 0) {
        const unsigned below_hi = (hi >= 32) ? 0xffffffffu : ((1u << hi) - 1u);
        const unsigned below_lo = (lo >= 32) ? 0xffffffffu : ((1u << lo) - 1u);
        pm = below_hi & ~below_lo;
    }
    // new rows: bit (k0 + kk - P) of the ancestor mask
    const int sh = k0 - P;
    unsigned nm;
    if (sh >= 128) nm = 0;
    else if (sh >= 64) nm = (unsigned)(b1 >> (sh - 64));
    else if (sh > 0) nm = (unsigned)((b0 >> sh) | (b1 << (64 - sh)));
    else if (sh == 0) nm = (unsigned)b0;
    else nm = (sh > -32) ? (unsigned)(b0 << (-sh)) : 0u;
    return pm | nm;
}

}  // namespace

}  // namespace tv
