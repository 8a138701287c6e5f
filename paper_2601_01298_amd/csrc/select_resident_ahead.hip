// Greedy landmark selection, register-resident, with the screen run AHEAD of time (bf16, d = 64, eight key rows
// per lane: the shape of a 32k-token head).
//
// Same method, same arithmetic and same exchange protocol as select_resident.hip, whose header describes them;
// read that first.  What differs: most of an exchange is waiting, and this kernel spends that time on the next
// step.  After an exchange every workgroup knows what the other workgroups proposed; the best proposal that did
// not win is, four times out of five, the winner of the NEXT exchange.  So between the two barriers of an
// exchange every wave fetches that landmark's row and screens its keys against it (the distances D are final at
// that point: they only change in the sweeps).  If the exchange then picks the expected landmark, the next sweep
// starts from the finished screen; if not, it screens as usual.  The screen never decides a value, so neither
// does the guess.  The per-lane results of the early screen wait in LDS; addresses derived from the thread id
// are rebuilt where they are used, because this shape leaves no register to carry them across the step loop.
#include "select_resident_common.h"
#include <type_traits>

namespace ws {

namespace {

using namespace resident;

// Workgroup barrier that orders LDS traffic only (global loads still in flight are not waited for).
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

struct Shared {
    unsigned dm[4], hi[4], lo[4];   // one entry per wave of the workgroup
    unsigned rdm, rhi, rlo;         // result of the exchange
    int pred;                       // runner-up among the workgroups' candidates of the last exchange (-1: none)
    int abort;
};

// One exchange over every wave of the head, carrying two independent maxima:
//   dm        a 32-bit value (D_max as float bits, or any other unsigned quantity);
//   (hi, lo)  a candidate compared as one 64-bit number, lo with its low 8 bits clear
//             (score bits, then the complemented index so that the lowest index wins ties).
// Three levels: lanes of a wave (done by the caller, the inputs are wave-uniform), the 4 waves of a
// workgroup through LDS, the workgroups of the head through two tagged 64-bit slots each in global
// memory.  Only wave 0 of a workgroup touches the slots: lanes 0 and 1 post, lane j polls slot A of
// member j and lane 32+j slot B, so a poll round of a whole head costs 2*nwg*nwg small requests at
// the L2 instead of (4 nwg)^2 * 16.  With `prefetch`, wave 0 touches the key row of this workgroup's
// candidate after posting, so that it is in this die's L2 when the winner is fetched.
// Returns false (for every thread of the workgroup) if the bounded wait expired.
template <class SpecIssue, class SpecRun>
__device__ __forceinline__ bool head_max(unsigned dm, unsigned hi, unsigned lo, Shared &sh, unsigned long long *gslots,
                                         int nwg, int member, unsigned &seq, unsigned &dm_out, unsigned &hi_out,
                                         unsigned &lo_out, const uint16_t *pf_base, int D, int last_row, bool prefetch,
                                         SpecIssue &&spec_issue, SpecRun &&spec_run)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));   // the same for every lane: branches on it are scalar
    if (lane == 0) {
        sh.dm[wave] = dm;
        sh.hi[wave] = hi;
        sh.lo[wave] = lo;
    }
    lds_barrier();
    // Between the two barriers most of an exchange is waiting.  That time goes into work for the NEXT step:
    // the screen against the landmark that is expected to win this exchange (the runner-up of the last one).
    const int pred = __builtin_amdgcn_readfirstlane(sh.pred);
    // The posting wave alternates with the half of the grid the workgroup is in: two workgroups share a CU,
    // and this keeps their posting waves off the same SIMD when they are dealt b and b + gridDim/2.
    const int pw = (blockIdx.x * 2 >= gridDim.x) ? 2 : 0;
    const bool poster = wave == pw && nwg > 1;       // the wave that posts and polls for the workgroup
    unsigned md = 0u, mh = 0u, ml = 0u, tag = 0u, touched = 0u;
    if (wave == pw) {
        // The exchange is the critical path of the step and this wave does more per step than the others: from
        // its first exchange on it goes first on its SIMD (a wave's own issue priority, nothing to do with streams).
        __builtin_amdgcn_s_setprio(3);
        // the 4 waves' entries: every lane reads all of them (same address: a broadcast), no cross-lane step
        md = max(max(sh.dm[0], sh.dm[1]), max(sh.dm[2], sh.dm[3]));
        mh = max(max(sh.hi[0], sh.hi[1]), max(sh.hi[2], sh.hi[3]));
#pragma unroll
        for (int w = 0; w < 4; ++w) ml = max(ml, sh.hi[w] == mh ? sh.lo[w] : 0u);
        md = (unsigned)__builtin_amdgcn_readfirstlane((int)md);
        mh = (unsigned)__builtin_amdgcn_readfirstlane((int)mh);
        ml = (unsigned)__builtin_amdgcn_readfirstlane((int)ml);
    }
    spec_issue(pred);       // its load goes out before the post and the touch, so it is back first
    if (poster) {
        ++seq;
        tag = seq % 255u + 1u;
        unsigned long long *slot = gslots + (seq & 1u) * 2 * kMaxMembers;   // [kind][member]
        // Per-lane addresses are rebuilt from the lane id on every call: kept live across the
        // whole step loop they would be spilled and reloaded on this, the latency-critical path.
        int ln = lane;
        asm volatile("" : "+v"(ln));
        post_words(slot, kMaxMembers, member, ln, md, mh, ml, tag);
        if (prefetch && ln < D / 8) {
            // candidate index travels in bits 8..31 of lo, complemented
            const int cand = min((int)(0xFFFFFFu - (ml >> 8)), last_row);
            touched = *reinterpret_cast<const unsigned *>(pf_base + (size_t)cand * D + ln * 8);
        }
    }
    spec_run(pred);         // while the touch and the others' posts are on their way
    unsigned keep_h = 0u, keep_l = 0u;      // poster: the candidate word this lane polled, for the next prediction
    bool good = true;
    if (poster) {
        asm volatile("" : "+v"(touched));       // the touch is waited for here: it also spaces the first poll from the post
        unsigned long long *slot = gslots + (seq & 1u) * 2 * kMaxMembers;
        int ln = lane;
        asm volatile("" : "+v"(ln));
        const int who = ln & 31, kind = ln >> 5;
        unsigned long long g = 0ull;
        good = poll_members(slot, kMaxMembers, nwg, ln, tag, g);
        if (who >= nwg || !good) g = 0ull;
        const unsigned gh = (unsigned)(g >> 32), gl = (unsigned)g & 0xFFFFFF00u;
        fold_polled(gh, gl, ln, md, mh, ml);
        keep_h = kind == 1 ? gh : 0u;
        keep_l = kind == 1 ? gl : 0u;
    }
    if (wave == pw && lane == 0) {
        sh.rdm = md;
        sh.rhi = mh;
        sh.rlo = ml;
        if (!good) sh.abort = 1;
    }
    lds_barrier();
    dm_out = sh.rdm;
    hi_out = sh.rhi;
    lo_out = sh.rlo;
    const bool fine = sh.abort == 0;
    if (wave == pw) {
        // The prediction for the next exchange: the best of the other workgroups' candidates.  (The true runner-up
        // may be the winning workgroup's second key; a prediction only has to be right most of the time.)
        int p = -1;
        if (poster) {
            const bool won = keep_h == mh && keep_l == ml;
            const unsigned xh = won ? 0u : keep_h, xl = won ? 0u : keep_l;
            const unsigned m2h = wave_umax(xh);
            const unsigned m2l = wave_pick_lo(xh == m2h && xl != 0u, xl);
            if (m2l != 0u) p = min((int)(0xFFFFFFu - (m2l >> 8)), last_row);
        }
        if (lane == 0) sh.pred = p;     // read after the next exchange's first barrier
    }
    return fine;
}

template <int D, int RREG, int RLDS>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
select_resident(ResArgs a)
{
    constexpr int R = RREG + RLDS;
    constexpr int DW = D / 2;      // 32-bit words per key row
    constexpr int NV = DW / 4;     // 16-byte pieces per key row
    __shared__ uint4 lrows[RLDS > 0 ? RLDS * NV * 256 : 1];
    __shared__ float nrm[R * 256];     // squared norm of every resident key (private to its thread)
    constexpr int LPK = DW / 2;              // lanes that share one staged key: 2 packed words (4 elements) each
    constexpr int KPP = 64 / LPK;            // staged keys a wave evaluates per pass (d = 64: four, d = 128: two)
    constexpr int CAP = (D == 64) ? 12 : 8;  // keys a wave can stage per step
    static_assert(CAP % KPP == 0, "whole passes");
    __shared__ __align__(16) uint32_t stage_all[4][CAP * DW];   // per wave: the packed rows of the staged keys
    __shared__ float sres_all[4][CAP];                          // per wave: the staged keys' exact distances
    __shared__ uint32_t spec_lmw_all[4][DW];      // per wave: the packed row of the landmark screened ahead of time
    __shared__ uint8_t spec_need_all[256];        // per lane: the row slots that screen flagged
    __shared__ Shared sh;

    int group, member;
    if ((a.groups & 7) == 0) {
        const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
        group = xcd * (a.groups >> 3) + j / a.wgpg;
        member = j % a.wgpg;
    } else {
        group = blockIdx.x / a.wgpg;
        member = blockIdx.x % a.wgpg;
    }
    int tid = threadIdx.x, lane = tid & 63;      // re-derived at every step (see the step loop)
    const int wv = member * 4 + (tid >> 6);
    if (tid == 0) {
        sh.abort = 0;
        sh.pred = -1;
    }
    __syncthreads();
    // Key blocks of 64 are dealt round-robin to the waves of the head: this lane's r-th key is
    // rowbase + rstride * r.  Neighbouring context positions tend to be neighbours in key space too, so
    // the keys a new landmark moves would otherwise pile up in one workgroup and make the others wait.
    const int rowbase = wv * 64 + lane;
    const int rstride = a.wgpg * 256;
    unsigned long long *gslots = a.slots + (size_t)group * 4 * kMaxMembers;
    const float alpha = a.alpha, oma = 1.0f - a.alpha;
    const float ninf = -__builtin_inff();
    unsigned seq = 0;

    for (int h = group; h < a.H; h += a.groups) {
        const uint16_t *Kh = a.K + (size_t)h * a.L * D;
        const float *rhoh = a.rho + (size_t)h * a.L;
        int t = 0;

        // ---- bring this lane's keys on chip, once per head
        uint32_t kr[RREG > 0 ? RREG : 1][DW];
#pragma unroll
        for (int r = 0; r < RREG; ++r) {
            const uint4 *p = reinterpret_cast<const uint4 *>(Kh + (size_t)min(rowbase + rstride * r, a.L - 1) * D);
#pragma unroll
            for (int c = 0; c < NV; ++c) {
                const uint4 q = p[c];
                kr[r][4 * c] = q.x;
                kr[r][4 * c + 1] = q.y;
                kr[r][4 * c + 2] = q.z;
                kr[r][4 * c + 3] = q.w;
            }
        }
#pragma unroll
        for (int r = 0; r < RLDS; ++r) {
            const uint4 *p = reinterpret_cast<const uint4 *>(Kh + (size_t)min(rowbase + rstride * (RREG + r), a.L - 1) * D);
#pragma unroll
            for (int c = 0; c < NV; ++c) lrows[(r * NV + c) * 256 + tid] = p[c];   // private to this thread
        }

        // ---- squared norms of the resident keys, for the screen below
#pragma unroll
        for (int r = 0; r < R; ++r) {
            float nn = 0.0f;
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
                    const bf16x2_t pr = __builtin_bit_cast(bf16x2_t, w4[j]);
                    nn = __builtin_amdgcn_fdot2_f32_bf16(pr, pr, nn, false);
                }
            }
            nrm[r * 256 + tid] = nn;
        }

        // ---- u_i = rho_min / rho_i ; keys past L count as already chosen
        float Dv[R], ou[R];
        float rmin = __builtin_inff();
        float rh[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int row = rowbase + rstride * r;
            rh[r] = rhoh[min(row, a.L - 1)];
            if (row < a.L) rmin = fminf(rmin, rh[r]);
        }
        {
            unsigned mdm, mhi, mlo;
            const unsigned mine = wave_umax(0xFFFFFFFFu - __float_as_uint(rmin));
            if (!head_max(mine, 0u, 0u, sh, gslots, a.wgpg, member, seq, mdm, mhi, mlo, Kh, D, a.L - 1, false, [](int) {},
                          [](int) {}))
                goto bail;
            rmin = __uint_as_float(0xFFFFFFFFu - mdm);
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const bool live = rowbase + rstride * r < a.L;
            Dv[r] = live ? __builtin_inff() : -1.0f;
            ou[r] = live ? oma * (rmin / rh[r]) : ninf;
        }

        {
            // Fetch of a landmark's row and the screen of every resident key against it, as one piece of code that
            // takes the landmark's index: it runs for the landmark just chosen and, ahead of time, for the one that is
            // expected next (see the exchange).
            auto fetch_screen = [&](int lm_idx, uint32_t (&lws)[DW], uint32_t &lmw, uint32_t &lmo, unsigned &needmask,
                                    unsigned &rowmask, float &ns, auto preloaded) {
                needmask = 0u;
                rowmask = 0u;
                // The landmark row is the same for every lane: read it through the constant address
                // space (K is never written while the kernel runs) so it arrives by scalar loads in
                // SGPRs and serves as a broadcast operand instead of occupying VGPRs.
                typedef const uint32_t __attribute__((address_space(4))) *cptr_t;
                const cptr_t lp = (cptr_t)(uintptr_t)(Kh + (size_t)lm_idx * D);
                // its squared norm: one packed pair per lane, summed over the wave
                // (lane l also keeps pair l mod D/2 of the landmark for the staged evaluation below)
                if (!decltype(preloaded)::value) {
                    int lx = tid;       // rebuilt here: the per-lane part of this address is not worth a register pair
                    asm volatile("" : "+v"(lx));
                    lmw = reinterpret_cast<const uint32_t *>(Kh + (size_t)lm_idx * D)[(lx & 63) % DW];
                }
                // (a) Screen.  Most keys are far from the new landmark and keep their D.  With
                // n = |k|^2, |k_i - s|^2 = n_i + n_s - 2 k_i.s, and the dot product runs on packed bf16
                // pairs (v_dot2c_f32_bf16: two elements per instruction, a sixth of the work of
                // widening, subtracting and squaring).  Its rounding and cancellation error is below
                // 2^-17 (n_i + n_s); a row slot goes on to an exact evaluation unless, for every lane,
                // the screened value exceeds D_i^2 by more than 2^-14 (n_i + n_s).  So the screen never
                // changes a result: it only skips evaluations that cannot lower D.
                // The packed landmark words are pinned in SGPRs for the whole step (the empty asm keeps
                // the compiler from re-fetching them in front of every row slot).
    #pragma unroll
                for (int i = 0; i < DW; ++i) lws[i] = lp[i];
                if (R > 4)      // one group of row slots reads them once anyway
    #pragma unroll
                for (int i = 0; i < DW; i += 16)
                    asm volatile(""
                                 : "+s"(lws[i]), "+s"(lws[i + 1]), "+s"(lws[i + 2]), "+s"(lws[i + 3]), "+s"(lws[i + 4]),
                                   "+s"(lws[i + 5]), "+s"(lws[i + 6]), "+s"(lws[i + 7]), "+s"(lws[i + 8]),
                                   "+s"(lws[i + 9]), "+s"(lws[i + 10]), "+s"(lws[i + 11]), "+s"(lws[i + 12]),
                                   "+s"(lws[i + 13]), "+s"(lws[i + 14]), "+s"(lws[i + 15]));
                // Row slots are screened four at a time so that four independent dot-product chains
                // interleave (one chain alone runs at the latency of the instruction, not its rate).
                // With rows parked in LDS a group is three register rows and one LDS row, whose 16-byte
                // pieces are read two pieces ahead of their use: the LDS latency hides behind the
                // dot products of two pieces instead of stalling every piece.
                constexpr bool MIX = RLDS > 0;   // groups of 3 + 1
                constexpr int NG = MIX ? RLDS : (R + 3) / 4;
                static_assert(!MIX || (RREG == 3 * RLDS), "a group is three register rows and one LDS row");
    #pragma unroll
                for (int g = 0; g < NG; ++g) {
                    // row slot behind position rr of this group (-1: none)
                    auto rowof = [&](int rr) -> int {
                        if (MIX) return rr < 3 ? 3 * g + rr : RREG + g;
                        return 4 * g + rr < R ? 4 * g + rr : -1;
                    };
                    float dot[4] = {0.0f, 0.0f, 0.0f, 0.0f};
                    uint4 pf[2];                 // LDS row: pieces c and c+1 in flight
                    if (MIX) {
                        pf[0] = lrows[(g * NV + 0) * 256 + tid];
                        __builtin_amdgcn_sched_barrier(0);
                    }
    #pragma unroll
                    for (int c = 0; c < NV; ++c) {
                        if (MIX) {
                            if (c + 1 < NV) pf[(c + 1) % 2] = lrows[(g * NV + c + 1) * 256 + tid];
                            __builtin_amdgcn_sched_barrier(0);
                        }
                        uint32_t w4[4][4];
    #pragma unroll
                        for (int rr = 0; rr < 4; ++rr) {
                            const int r = rowof(rr);
                            if (r >= 0 && r < RREG) {
                                w4[rr][0] = kr[r >= 0 && r < RREG ? r : 0][4 * c];
                                w4[rr][1] = kr[r >= 0 && r < RREG ? r : 0][4 * c + 1];
                                w4[rr][2] = kr[r >= 0 && r < RREG ? r : 0][4 * c + 2];
                                w4[rr][3] = kr[r >= 0 && r < RREG ? r : 0][4 * c + 3];
                            } else if (r >= 0) {
                                const uint4 q = pf[c % 2];
                                w4[rr][0] = q.x;
                                w4[rr][1] = q.y;
                                w4[rr][2] = q.z;
                                w4[rr][3] = q.w;
                            } else {
                                w4[rr][0] = w4[rr][1] = w4[rr][2] = w4[rr][3] = 0u;
                            }
                        }
    #pragma unroll
                        for (int j = 0; j < 4; ++j)
    #pragma unroll
                            for (int rr = 0; rr < 4; ++rr)
                                if (rowof(rr) >= 0)
                                    dot[rr] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w4[rr][j]),
                                                                              __builtin_bit_cast(bf16x2_t, lws[4 * c + j]),
                                                                              dot[rr], false);
                        if (MIX) __builtin_amdgcn_sched_barrier(0);
                    }
                    if (g == 0) {
                        // the landmark's own squared norm: one packed pair per lane, summed over the wave
                        // (used only now, so the vector load above overlaps the first dot-product chains)
                        float nsp = 0.0f;
                        if (lane < DW) {
                            const bf16x2_t lw = __builtin_bit_cast(bf16x2_t, lmw);
                            nsp = __builtin_amdgcn_fdot2_f32_bf16(lw, lw, 0.0f, false);
                        }
                        ns = wave_fsum(nsp);
                        {   // for the staged evaluation: the other packed word, from the lane LPK further on (the lane
                            // id is rebuilt here: kept across the step loop it ends up in scratch)
                            int lx = tid;
                            asm volatile("" : "+v"(lx));
                            lmo = (uint32_t)__builtin_amdgcn_ds_bpermute(((lx & 63) ^ LPK) << 2, (int)lmw);
                        }
                    }
    #pragma unroll
                    for (int rr = 0; rr < 4; ++rr) {
                        const int r = rowof(rr);
                        if (r >= 0) {
                            const float nsum = nrm[r * 256 + tid] + ns;
                            const float d2a = fmaf(-2.0f, dot[rr], nsum);
                            const bool need = fmaf(nsum, -6.103515625e-5f, d2a) < Dv[r] * Dv[r];
                            const int cnt = __popcll(__ballot(need));
                            if (need) needmask |= 1u << r;
                            if (cnt > 0) rowmask |= 1u << r;
                        }
                    }
                }
            };

            // What the screen found for the landmark that was expected to win (spec_idx; -1: nothing at hand).
            int spec_idx = -1;
            unsigned spec_rows = 0u;          // the same in every lane, like spec_ns; the per-lane results wait in LDS
            float spec_ns = 0.0f;
            uint32_t spec_lmw = 0u;           // in flight between the two halves of the speculative work only
            auto spec_issue = [&](int pred) {
                if (pred >= 0 && spec_idx < 0)
                    spec_lmw = reinterpret_cast<const uint32_t *>(Kh + (size_t)pred * D)[lane % DW];
            };
            auto spec_run = [&](int pred) {
                if (pred >= 0 && spec_idx < 0) {
                    uint32_t lws2[DW], lmo2;
                    unsigned need2, rows2;
                    float ns2;
                    fetch_screen(pred, lws2, spec_lmw, lmo2, need2, rows2, ns2, std::true_type{});
                    spec_ns = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(ns2)));
                    spec_rows = (unsigned)__builtin_amdgcn_readfirstlane((int)rows2);
                    spec_need_all[tid] = (uint8_t)need2;
                    if (lane < DW) spec_lmw_all[tid >> 6][lane] = spec_lmw;
                    spec_idx = pred;
                }
            };
            int prev = 0;
            unsigned dprev = 0xFFFFFFFFu;    // bits of the D_max the last step ended with (none yet)
            for (t = 0; t < a.k; ++t) {
                unsigned lbits = 0u;
                if (t > 0) {
                    // ---- distance of every resident key to landmark `prev`: fetch of its row, then the screen.
                    // Both sit in one piece of code that takes the landmark's index, so that it can also run ahead
                    // of time for a landmark that is only expected (see the exchange below).
                    unsigned needmask = 0u;          // bit r: this lane's key of row slot r may move
                    unsigned rowmask = 0u;           // bit r: some key of row slot r may move (wave-uniform)
                    float ns = 0.0f;                 // squared norm of the landmark (set once its pair has arrived)
                    uint32_t lmo = 0u, lmw = 0u;
                    uint32_t lws[DW];
                    unsigned sh16 = 16u, mhi16 = 0xFFFF0000u;
                    asm volatile("" : "+s"(sh16), "+s"(mhi16));
                    if (prev == spec_idx) {
                        // the winner is the landmark that was screened while the exchange was under way
                        int tx = tid;
                        asm volatile("" : "+v"(tx));
                        lmw = spec_lmw_all[tx >> 6][(tx & 63) % DW];
                        lmo = (uint32_t)__builtin_amdgcn_ds_bpermute(((tx & 63) ^ LPK) << 2, (int)lmw);
                        ns = spec_ns;
                        needmask = spec_need_all[tx];
                        rowmask = spec_rows;
#pragma unroll
                        for (int i = 0; i < DW; ++i) lws[i] = (uint32_t)__builtin_amdgcn_readlane((int)lmw, i);
                    } else {
                        fetch_screen(prev, lws, lmw, lmo, needmask, rowmask, ns, std::false_type{});
                    }
                    spec_idx = -1;
                    // the wave's strips are located afresh in every step: kept across the step loop their addresses
                    // end up in scratch
                    int wl = tid >> 6;
                    asm volatile("" : "+v"(wl));
                    lbits = exact_update<D, RREG, RLDS, CAP>(kr, lrows, lws, Dv, needmask, rowmask, stage_all[wl], sres_all[wl], tid,
                                                            lane, lmw, lmo, sh16, mhi16);
                }

                int s;
                float sc;
                if (t == 0 && alpha == 1.0f) {
                    s = 0;
                    sc = alpha;
                } else {
                    // ---- score = alpha * D/D_max + (1-alpha) * u ; keys in ascending order per lane.
                    // First with the D_max of the previous step (step 0: coverage term 1 for every key),
                    // sent together with this step's local D maximum; again only if D_max moved.
                    unsigned mdm = 0u, mhi = 0u, mlo = 0u;
                    for (int pass = 0; pass < 2; ++pass) {
                        const float dmax = __uint_as_float(dprev);
                        const float ainv = (t == 0) ? alpha : (dmax > 0.0f ? alpha / dmax : 0.0f);
                        float best = -1.0f;
                        int bi = 0;
#pragma unroll
                        for (int r = 0; r < R; ++r) {
                            const float dd = (t == 0) ? 1.0f : Dv[r];
                            const float v = fmaf(ainv, dd, ou[r]);
                            if (v > best) {
                                best = v;
                                bi = rowbase + rstride * r;
                            }
                        }
                        const unsigned chi = best >= 0.0f ? __float_as_uint(best) : 0u;
                        const unsigned clo = best >= 0.0f ? (0xFFFFFFu - (unsigned)bi) << 8 : 0u;
                        const unsigned whi = wave_umax(chi);
                        const unsigned wlo = wave_pick_lo(chi == whi, clo);
                        if (!head_max(lbits, whi, wlo, sh, gslots, a.wgpg, member, seq, mdm, mhi, mlo, Kh, D, a.L - 1, true,
                                      spec_issue, spec_run))
                            goto bail;
                        if (t == 0 || mdm == dprev) break;     // the guess was the true D_max
                        dprev = mdm;
                    }
                    s = min((int)(0xFFFFFFu - (mlo >> 8)), a.L - 1);   // in range whatever the inputs held
                    sc = __uint_as_float(mhi);
                }
                s = __builtin_amdgcn_readfirstlane(s);
                if (wv == 0 && lane == 0) {
                    a.idx[(size_t)h * a.k + t] = s;
                    if (a.score_out) a.score_out[(size_t)h * a.k + t] = sc;
                }
#pragma unroll
                for (int r = 0; r < R; ++r)
                    if (rowbase + rstride * r == s) {       // chosen: never scored again
                        Dv[r] = -1.0f;
                        ou[r] = ninf;
                    }
                prev = s;
            }
        }
        continue;
    bail:
        if (lane == 0) atomicExch(a.fail, 1);
        if (wv == 0) {
            for (int hh = h; hh < a.H; hh += a.groups) {
                const int t0 = (hh == h) ? t : 0;
                for (int tt = t0 + lane; tt < a.k; tt += 64) a.idx[(size_t)hh * a.k + tt] = -1;
            }
        }
        return;
    }
}


template <int D, int RREG, int RLDS>
hipError_t run(const ResArgs &a, hipStream_t st)
{
    hipLaunchKernelGGL((select_resident<D, RREG, RLDS>), dim3(a.groups * a.wgpg), dim3(256), 0, st, a);
    return hipGetLastError();
}

}  // namespace

hipError_t resident_ahead_occupancy(int *workgroups_per_cu)
{
    return hipOccupancyMaxActiveBlocksPerMultiprocessor(workgroups_per_cu, select_resident<64, 6, 2>, 256, 0);
}

// The caller (launch_select_resident) has chosen the shape, laid out the workspace and cleared slots and flag.
hipError_t launch_select_resident_ahead(const void *K, int H, int L, const float *rho, int k, float alpha, int32_t *idx,
                                        float *score_out, unsigned long long *slots, int *fail, int groups, int wgpg,
                                        hipStream_t st)
{
    ResArgs a;
    a.K = reinterpret_cast<const uint16_t *>(K);
    a.rho = rho;
    a.idx = idx;
    a.score_out = score_out;
    a.slots = slots;
    a.fail = fail;
    a.H = H;
    a.L = L;
    a.k = k;
    a.groups = groups;
    a.wgpg = wgpg;
    a.alpha = alpha;
    return run<64, 6, 2>(a, st);
}

}  // namespace ws
