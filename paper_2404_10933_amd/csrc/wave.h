// Wave-level (64 lanes, gfx950) helpers: DPP scans and reductions on 64-bit
// integers, lane broadcast, and exact division of 63-bit values by a small
// divisor through a multiply-high.
#pragma once

#ifndef __HIPCC_RTC__
#include <hip/hip_runtime.h>
#include <stdint.h>
#endif

namespace llmem {

typedef unsigned long long u64;
typedef long long i64;
typedef unsigned int u32;

__device__ __forceinline__ int lane_id() { return (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u)); }

// Orders the LDS accesses of this wavefront's lanes among themselves: what any lane wrote before
// this point is what every lane reads after it, and no read from before it is moved behind a
// write after it.  A wavefront executes its LDS instructions in order, so this costs no
// instruction; it keeps the compiler from reordering or merging across the point.
__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// DPP controls of the GFX9 family
enum : int {
    DPP_ROW_SHR1 = 0x111, DPP_ROW_SHR2 = 0x112, DPP_ROW_SHR4 = 0x114, DPP_ROW_SHR8 = 0x118,
    DPP_ROW_BCAST15 = 0x142, DPP_ROW_BCAST31 = 0x143,
};

// Value of `v` in the lane selected by the DPP control; lanes with no source
// lane, or outside row_mask, get `fill`.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ i64 dpp_fetch(i64 v, i64 fill)
{
    int lo = __builtin_amdgcn_update_dpp((int)(u32)(u64)fill, (int)(u32)(u64)v, CTRL, ROW_MASK, 0xf, false);
    int hi = __builtin_amdgcn_update_dpp((int)((u64)fill >> 32), (int)((u64)v >> 32), CTRL, ROW_MASK, 0xf, false);
    return (i64)(((u64)(u32)hi << 32) | (u64)(u32)lo);
}

// Inclusive prefix sum over the 64 lanes.
__device__ __forceinline__ i64 wave_scan_add(i64 v)
{
    v += dpp_fetch<DPP_ROW_SHR1, 0xf>(v, 0);
    v += dpp_fetch<DPP_ROW_SHR2, 0xf>(v, 0);
    v += dpp_fetch<DPP_ROW_SHR4, 0xf>(v, 0);
    v += dpp_fetch<DPP_ROW_SHR8, 0xf>(v, 0);
    v += dpp_fetch<DPP_ROW_BCAST15, 0xa>(v, 0);
    v += dpp_fetch<DPP_ROW_BCAST31, 0xc>(v, 0);
    return v;
}

__device__ __forceinline__ i64 max64(i64 a, i64 b) { return a > b ? a : b; }

// Inclusive prefix maximum over the 64 lanes.
__device__ __forceinline__ i64 wave_scan_max(i64 v)
{
    const i64 lowest = (i64)0x8000000000000000ull;
    v = max64(v, dpp_fetch<DPP_ROW_SHR1, 0xf>(v, lowest));
    v = max64(v, dpp_fetch<DPP_ROW_SHR2, 0xf>(v, lowest));
    v = max64(v, dpp_fetch<DPP_ROW_SHR4, 0xf>(v, lowest));
    v = max64(v, dpp_fetch<DPP_ROW_SHR8, 0xf>(v, lowest));
    v = max64(v, dpp_fetch<DPP_ROW_BCAST15, 0xa>(v, lowest));
    v = max64(v, dpp_fetch<DPP_ROW_BCAST31, 0xc>(v, lowest));
    return v;
}

// Value of a 64-bit register in one (wave-uniform) lane, as a wave-uniform value.
__device__ __forceinline__ i64 read_lane(i64 v, int lane)
{
    u32 lo = (u32)__builtin_amdgcn_readlane((int)(u32)(u64)v, lane);
    u32 hi = (u32)__builtin_amdgcn_readlane((int)((u64)v >> 32), lane);
    return (i64)(((u64)hi << 32) | lo);
}
__device__ __forceinline__ u32 read_lane(u32 v, int lane) { return (u32)__builtin_amdgcn_readlane((int)v, lane); }

// Put a value into lane `lane` of `acc` (`me` = this lane's id).
__device__ __forceinline__ i64 write_lane(i64 acc, i64 value, int lane, int me)
{
    return me == lane ? value : acc;
}
__device__ __forceinline__ u32 write_lane(u32 acc, u32 value, int lane, int me)
{
    return me == lane ? value : acc;
}

__device__ __forceinline__ i64 wave_sum(i64 v) { return read_lane(wave_scan_add(v), 63); }
__device__ __forceinline__ i64 wave_max(i64 v) { return read_lane(wave_scan_max(v), 63); }

// ---------------------------------------------------------------------------
// x / d for 0 <= x < 2^63 and 1 <= d <= 255 without a hardware divide:
// q = mulhi64(x, M[d]) >> S[d], with M[d] = ceil(2^(63+l) / d), l = ceil(log2 d),
// S[d] = l - 1 (Granlund-Montgomery round-up method; exact because the numerator
// has at most 63 bits).  d = 1 is passed through.
// ---------------------------------------------------------------------------
struct DivMagic { u64 mul; u32 shift; };

constexpr DivMagic make_magic(unsigned d)
{
    if (d < 2) return DivMagic{0, 0};
    unsigned l = 0;
    while ((1u << l) < d) ++l;
    unsigned __int128 num = (unsigned __int128)1 << (63 + l);
    unsigned __int128 m = (num + d - 1) / d;
    return DivMagic{(u64)m, l - 1};
}

struct DivMagicTable {
    DivMagic t[256];
    constexpr DivMagicTable() : t{} { for (unsigned d = 0; d < 256; ++d) t[d] = make_magic(d); }
};

// one copy per translation unit (device symbols are not shared across them)
static __constant__ DivMagicTable c_div = DivMagicTable();

}  // namespace llmem
