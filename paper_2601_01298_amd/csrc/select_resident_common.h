// Pieces shared by the two register-resident selection kernels (select_resident.hip and
// select_resident_ahead.hip): the launch arguments, the exchange protocol between the workgroups
// of a head (its limits, the post, the poll of up to 32 members, the fold of what was polled), the
// pass over a wave's staged keys, and the wave-level reductions both step loops are built from.
// The step loops themselves, and what each kernel does between post and poll, stay in their own
// files: the eight-rows-per-lane instance sits exactly at its register budget and is laid out by
// hand.
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

// ---- the exchange between the workgroups of a head ---------------------------------------------------------
// Every workgroup owns two tagged 64-bit slots per phase, [kind][member]: kind 0 carries its D maximum
// (value << 32 | tag), kind 1 its candidate (score bits << 32 | complemented index << 8 | tag).  One wave per
// workgroup posts and polls; `ln` is that wave's lane id (rebuilt by the caller behind an empty statement, so the
// addresses derived from it do not stay in registers across the step loop).

// lanes 0 and 1 of the posting wave write the workgroup's two words
__device__ __forceinline__ void post_words(unsigned long long *slot, int slots_per_kind, int member, int ln, unsigned md,
                                           unsigned mh, unsigned ml, unsigned tag)
{
    if (ln < 2) {
        const unsigned long long word =
            ln == 0 ? (((unsigned long long)md << 32) | tag) : (((unsigned long long)mh << 32) | ml | tag);
        __hip_atomic_store(slot + ln * slots_per_kind + member, word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// Up to 32 members: lane j polls the D maximum of member j, lane 32 + j its candidate, until every word carries
// this exchange's tag or the bounded wait expires (returns false).  g: the word this lane polled.
__device__ __forceinline__ bool poll_members(const unsigned long long *slot, int slots_per_kind, int nwg, int ln,
                                             unsigned tag, unsigned long long &g)
{
    const int who = ln & 31, kind = ln >> 5;
    bool ok = who >= nwg;
    unsigned spins = 0;
    g = 0ull;
    while (true) {
        if (!ok) {
            g = __hip_atomic_load(slot + kind * slots_per_kind + who, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            ok = (unsigned)(g & 0xFFull) == tag;
        }
        if (__all(ok)) return true;
        if (++spins > kSpinLimit) return false;
        if (spins > 16) __builtin_amdgcn_s_sleep(1);
    }
}

// Fold of the polled words (high halves gh, low halves gl with the tag cleared; 0 in lanes without a member): lanes
// 0..31 hold D maxima, lanes 32..63 candidates, so one row-wise pass serves both; the candidate's low half comes from
// the lane whose high half won.
__device__ __forceinline__ void fold_polled(unsigned gh, unsigned gl, int ln, unsigned &md, unsigned &mh, unsigned &ml)
{
    unsigned v = gh;
    v = dpp_umax<0xB1>(v);
    v = dpp_umax<0x4E>(v);
    v = dpp_umax<0x141>(v);
    v = dpp_umax<0x140>(v);
    const unsigned r0 = (unsigned)__builtin_amdgcn_readlane((int)v, 0);
    const unsigned r1 = (unsigned)__builtin_amdgcn_readlane((int)v, 16);
    const unsigned r2 = (unsigned)__builtin_amdgcn_readlane((int)v, 32);
    const unsigned r3 = (unsigned)__builtin_amdgcn_readlane((int)v, 48);
    md = r0 > r1 ? r0 : r1;
    mh = r2 > r3 ? r2 : r3;
    ml = wave_pick_lo((ln >> 5) == 1 && gh == mh, gl);
}

// ---- the staged keys of a wave ---------------------------------------------------------------------------------
// `total` packed key rows (DW words each) wait in the wave's strip `stage`; their exact distances to the landmark go to
// `sres`.  KPP = 64 / LPK keys per pass: LPK = DW / 2 lanes share a key, each takes two packed words of it (from the
// strip) and of the landmark row (lmw: the word this lane already holds, lmo: the one the lane LPK further on holds),
// direct differences in fp32, then the partial sums of a key meet by DPP inside their lane group.  No barrier and no
// atomic: key blocks are dealt round-robin, so the waves of a head stage about the same number of keys.  Slots past
// `total` hold stale rows: computed, never used.
template <int DW>
__device__ __forceinline__ void evaluate_staged(const uint32_t *stage, float *sres, int total, int lane, uint32_t lmw,
                                                uint32_t lmo)
{
    constexpr int LPK = DW / 2;
    constexpr int KPP = 64 / LPK;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    // lane-derived addresses are rebuilt here every step: hoisted out of the step loop they would occupy registers
    // that the resident keys need
    int ln = lane;
    asm volatile("" : "+v"(ln));
    const int sub = ln / LPK, part = ln % LPK;
    const bool odd = (sub & 1) != 0;
    const uint32_t wa = odd ? lmo : lmw, wb = odd ? lmw : lmo;
    const float l0 = __uint_as_float(wa << 16), l1 = __uint_as_float(wa & 0xFFFF0000u);
    const float l2 = __uint_as_float(wb << 16), l3 = __uint_as_float(wb & 0xFFFF0000u);
    for (int q0 = 0; q0 < total; q0 += KPP) {
        const uint32_t ka = stage[(q0 + sub) * DW + part], kb = stage[(q0 + sub) * DW + part + LPK];
        const float d0 = __uint_as_float(ka << 16) - l0, d1 = __uint_as_float(ka & 0xFFFF0000u) - l1;
        const float d2 = __uint_as_float(kb << 16) - l2, d3 = __uint_as_float(kb & 0xFFFF0000u) - l3;
        float pr = fmaf(d1, d1, d0 * d0) + fmaf(d3, d3, d2 * d2);
        pr = dpp_fadd<0xB1>(pr);
        pr = dpp_fadd<0x4E>(pr);
        pr = dpp_fadd<0x141>(pr);
        pr = dpp_fadd<0x140>(pr);          // every lane: the sum over its row of 16
        if (LPK == 16) {
            if (part == 0) sres[q0 + sub] = __fsqrt_rn(pr);
        } else {
            const float s0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(pr), 0));
            const float s1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(pr), 16));
            const float s2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(pr), 32));
            const float s3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(pr), 48));
            if (ln < 2) sres[q0 + ln] = __fsqrt_rn(ln == 0 ? s0 + s1 : s2 + s3);
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// ---- exact distances for the keys a new landmark may move ------------------------------------------------------
// After the screen: bit r of `rowmask` says some key of row slot r may move (wave-uniform), bit r of `needmask` that
// this lane's key of the slot may.  kr: the lane's rows held in registers (packed bf16 pairs), lrows: its rows in
// LDS, lws: the landmark row (scalar registers), Dv: the lane's distances, updated in place.  sh16 / mhi16: 16 and
// 0xFFFF0000 passed through an empty statement by the caller, so that the widened keys are not treated as loop
// invariants.  Returns the bits of the wave's largest distance afterwards.
// (Bringing the keys on chip, the step before this in both kernels, stays written out in each of them: as a shared
// function it changes the register allocation of the eight-rows-per-lane instances, 21 -> 33 spilled registers.)
template <int D, int RREG, int RLDS, int CAP>
__device__ __forceinline__ unsigned exact_update(const uint32_t (&kr)[RREG > 0 ? RREG : 1][D / 2], const uint4 *lrows,
                                                 const uint32_t (&lws)[D / 2], float (&Dv)[RREG + RLDS], unsigned needmask,
                                                 unsigned rowmask, uint32_t *stage, float *sres, int tid, int lane,
                                                 uint32_t lmw, uint32_t lmo, unsigned sh16, unsigned mhi16)
{
    constexpr int R = RREG + RLDS;
    constexpr int DW = D / 2;          // packed bf16 pairs per key row
    constexpr int NV = D / 8;          // 16-byte pieces per key row
    // row slots whose keys no longer fit the wave's staging strip (the first steps, when most keys move) are
    // evaluated whole instead
    int base = 0;
                        unsigned pm0 = 0u, pm1 = 0u;     // per row slot, 1 + the staging position of this lane's key
                        float lmax;
                        unsigned stmask = 0u;            // bit r: row slot r has keys in the staging area (wave-uniform)
                        rowmask = __builtin_amdgcn_readfirstlane(rowmask);
    #pragma unroll
                        for (int r = 0; r < R; ++r) {
                            if (!(rowmask & (1u << r))) continue;
                            const bool need = (needmask >> r) & 1u;
                            const unsigned long long bal = __ballot(need);
                            const int cnt = __popcll(bal);
                            if (cnt <= CAP - base) {
                                stmask |= 1u << r;
                                // (b) A few keys of the slot may move (the usual case: about 1 % of all keys per
                                // step): their owners copy the packed rows to the wave's staging strip.
                                const int pos = base + (int)__builtin_amdgcn_mbcnt_hi((unsigned)(bal >> 32),
                                                                                      __builtin_amdgcn_mbcnt_lo((unsigned)bal, 0u));
                                base += cnt;
                                if (need) {
    #pragma unroll
                                    for (int c = 0; c < NV; ++c) {
                                        uint4 q;
                                        if (r < RREG) {
                                            q = make_uint4(kr[r < RREG ? r : 0][4 * c], kr[r < RREG ? r : 0][4 * c + 1],
                                                           kr[r < RREG ? r : 0][4 * c + 2], kr[r < RREG ? r : 0][4 * c + 3]);
                                        } else {
                                            q = lrows[((r - RREG) * NV + c) * 256 + tid];
                                        }
                                        *reinterpret_cast<uint4 *>(&stage[pos * DW + 4 * c]) = q;
                                        if (r >= RREG) __builtin_amdgcn_sched_barrier(0);
                                    }
                                    if (r < 4) pm0 |= (unsigned)(pos + 1) << (8 * (r & 3));
                                    else pm1 |= (unsigned)(pos + 1) << (8 * (r & 3));
                                }
                            } else {
                                // (c) Many keys of the slot may move: the whole slot, each lane its own key,
                                // direct coordinate differences in fp32.
                                float acc = 0.0f;
    #pragma unroll
                                for (int c = 0; c < NV; ++c) {
                                    uint32_t w4[4];
                                    if (r < RREG) {
                                        w4[0] = kr[r < RREG ? r : 0][4 * c];
                                        w4[1] = kr[r < RREG ? r : 0][4 * c + 1];
                                        w4[2] = kr[r < RREG ? r : 0][4 * c + 2];
                                        w4[3] = kr[r < RREG ? r : 0][4 * c + 3];
                                    } else {
                                        const uint4 q = lrows[((r - RREG) * NV + c) * 256 + tid];
                                        w4[0] = q.x;
                                        w4[1] = q.y;
                                        w4[2] = q.z;
                                        w4[3] = q.w;
                                    }
    #pragma unroll
                                    for (int j = 0; j < 4; ++j) {
                                        const uint32_t wd = lws[4 * c + j];
                                        const float d0 = __uint_as_float(w4[j] << sh16) - __uint_as_float(wd << 16);
                                        acc = fmaf(d0, d0, acc);
                                        const float d1 = __uint_as_float(w4[j] & mhi16) - __uint_as_float(wd & 0xFFFF0000u);
                                        acc = fmaf(d1, d1, acc);
                                    }
                                    if (r >= RREG) __builtin_amdgcn_sched_barrier(0);
                                }
                                Dv[r] = fminf(Dv[r], __fsqrt_rn(acc));    // chosen keys stay at -1
                            }
                        }
                        // ---- the staged keys of this wave: exact distances, several keys per pass (evaluate_staged)
                        const int total = base;
                        if (total > 0) {
                            evaluate_staged<DW>(stage, sres, total, lane, lmw, lmo);
    #pragma unroll
                            for (int r = 0; r < R; ++r) {
                                if (stmask & (1u << r)) {
                                    const unsigned pb = ((r < 4 ? pm0 : pm1) >> (8 * (r & 3))) & 0xFFu;
                                    const float dn = sres[pb ? pb - 1 : 0];
                                    if (pb) Dv[r] = fminf(Dv[r], dn);    // chosen keys stay at -1
                                }
                            }
                        }
                        lmax = 0.0f;
    #pragma unroll
                        for (int r = 0; r < R; ++r) lmax = fmaxf(lmax, Dv[r]);
                        return wave_umax(__float_as_uint(lmax));
}

}  // namespace resident
}  // namespace ws
