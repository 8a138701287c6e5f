// Pieces shared by the two register-resident selection kernels (select_resident.hip and
// select_resident_ahead.hip): the launch arguments, the limits of the exchange protocol, and the
// wave-level reductions both step loops are built from.  The step loops themselves stay in their
// own files: the eight-rows-per-lane instance sits exactly at its register budget and is laid out
// by hand.
#pragma once
#include "ws_internal.h"

namespace ws {
namespace resident {

constexpr int kMaxMembers = 32;             // workgroups cooperating on one head (one slot polled per lane) ...
constexpr int kMaxMembersWide = 128;        // ... and in the wide instances for heads that need more (four per lane)
constexpr unsigned kSpinLimit = 1u << 22;

struct ResArgs {
    const uint16_t *K;
    const float *rho;
    int32_t *idx;
    float *score_out;
    unsigned long long *slots;   // [groups][2 phases][2 kinds][kMaxMembers, or kMaxMembersWide in a wide instance]
    int *fail;
    int H, L, k;
    int groups, wgpg;            // heads in flight, workgroups per head
    float alpha;
};

// ---- wave-wide unsigned max via DPP: 4 in-row steps, then one lane of each 16-lane row ------
template <int CTRL>
__device__ __forceinline__ unsigned dpp_umax(unsigned v)
{
    const unsigned o = (unsigned)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, 0xF, 0xF, false);
    return o > v ? o : v;
}

__device__ __forceinline__ unsigned wave_umax(unsigned v)
{
    v = dpp_umax<0xB1>(v);    // quad_perm [1,0,3,2]
    v = dpp_umax<0x4E>(v);    // quad_perm [2,3,0,1]
    v = dpp_umax<0x141>(v);   // row_half_mirror
    v = dpp_umax<0x140>(v);   // row_mirror
    const unsigned a = (unsigned)__builtin_amdgcn_readlane((int)v, 0);
    const unsigned b = (unsigned)__builtin_amdgcn_readlane((int)v, 16);
    const unsigned c = (unsigned)__builtin_amdgcn_readlane((int)v, 32);
    const unsigned d = (unsigned)__builtin_amdgcn_readlane((int)v, 48);
    const unsigned ab = a > b ? a : b, cd = c > d ? c : d;
    return ab > cd ? ab : cd;
}

// wave-wide float sum; every lane ends up with the same value
template <int CTRL>
__device__ __forceinline__ float dpp_fadd(float v)
{
    return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}

__device__ __forceinline__ float wave_fsum(float v)
{
    v = dpp_fadd<0xB1>(v);
    v = dpp_fadd<0x4E>(v);
    v = dpp_fadd<0x141>(v);
    v = dpp_fadd<0x140>(v);
    const float a = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
    const float b = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
    const float c = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
    const float d = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
    return (a + b) + (c + d);
}

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

// Second half of a 64-bit maximum over the wave: `lo` of the lane whose first half matched.  Nearly
// always exactly one lane matches, and then a ballot and one readlane replace the whole reduction.
__device__ __forceinline__ unsigned wave_pick_lo(bool match, unsigned lo)
{
    const unsigned long long m = __ballot(match);
    if (__popcll(m) == 1) return (unsigned)__builtin_amdgcn_readlane((int)lo, (int)__builtin_ctzll(m));
    return wave_umax(match ? lo : 0u);
}

}  // namespace resident
}  // namespace ws
