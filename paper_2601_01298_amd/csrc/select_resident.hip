// Greedy landmark selection, register-resident variant (bf16 keys).
//
// The selection makes k dependent sweeps over the same L keys of a head (Warp-Cortex Sec. 3.3:
// one landmark per step, each step needs every key's distance to the landmark just chosen).
// Streaming those keys from HBM k times costs k*L*d*2 bytes per head; but the register files
// and LDS of the chip together hold ~100 MB, so a few dozen heads at a time fit ON CHIP.  Here
// every wave owns 64*R keys for the whole life of a head: lane l keeps R complete key rows
// (RREG of them in VGPRs, RLDS in a private strip of LDS), its D and u values, and never
// touches HBM again until the next head.  Blocks of 64 keys are dealt round-robin to the waves of
// the head.  The landmark row is fetched once per step through the scalar cache into SGPRs and
// used as a broadcast operand.
//
// Only about 1 % of the keys get closer to the chosen set in a step.  A dot-product screen on the
// packed bf16 pairs (|k-s|^2 = |k|^2 + |s|^2 - 2 k.s, v_dot2c_f32_bf16) with a proven error margin
// finds the keys that cannot move; the rest are evaluated exactly, by direct differences in fp32:
// their owners copy the rows to a staging strip of the wave, which then evaluates them a few per
// pass (d = 64: four, 16 lanes sharing a key), each lane two packed pairs.  The screen only skips
// work, it never decides a value.
//
// A head is shared by up to 32 workgroups of 4 waves, placed on one accelerator die.  A step needs
// two maxima over all keys of the head, the second depending on the first: D_max, then the best
// score alpha*D/D_max + (1-alpha)*u.  D_max rarely changes from one step to the next (the far
// point that sets it stays uncovered for long stretches), so every workgroup scores its keys with
// the PREVIOUS step's D_max and sends its local D maximum and its candidate in ONE exchange; only
// when the new D_max differs from the guess are the candidates recomputed and exchanged again
// (same arithmetic either way, so the picks do not depend on the guess).  An exchange reduces in
// three levels: lanes of a wave with DPP row operations, the waves of a workgroup through LDS, and
// the workgroups of the head through two tagged 64-bit slots each in global memory, posted and
// polled by a single wave per workgroup (keeping the number of requests that hit the slots' L2
// channel small matters more than saving a barrier).  Waits are bounded; a workgroup whose wait
// expires raises the failure flag, and (if it is the head's writer) writes -1 into the index entries
// still owed, then leaves.
#include "select_resident_common.h"

namespace ws {

namespace {

using namespace resident;

struct Shared {
    unsigned dm[4], hi[4], lo[4];   // one entry per wave of the workgroup
    unsigned rdm, rhi, rlo;         // result of the exchange
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
template <bool WIDE>
__device__ __forceinline__ bool head_max(unsigned dm, unsigned hi, unsigned lo, Shared &sh, unsigned long long *gslots,
                                         int nwg, int member, unsigned &seq, unsigned &dm_out, unsigned &hi_out,
                                         unsigned &lo_out, const uint16_t *pf_base, int D, int last_row, bool prefetch)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) {
        sh.dm[wave] = dm;
        sh.hi[wave] = hi;
        sh.lo[wave] = lo;
    }
    __syncthreads();
    if (wave == 0) {
        // The exchange is the critical path of the step: from its first exchange on, the wave that carries it goes
        // first on its SIMD (a wave's own issue priority).
        __builtin_amdgcn_s_setprio(3);
        // the 4 waves' entries: every lane reads all of them (same address: a broadcast), no cross-lane step
        unsigned md = max(max(sh.dm[0], sh.dm[1]), max(sh.dm[2], sh.dm[3]));
        unsigned mh = max(max(sh.hi[0], sh.hi[1]), max(sh.hi[2], sh.hi[3]));
        unsigned ml = 0u;
#pragma unroll
        for (int w = 0; w < 4; ++w) ml = max(ml, sh.hi[w] == mh ? sh.lo[w] : 0u);
        bool good = true;
        if (nwg > 1) {
            ++seq;
            const unsigned tag = seq % 255u + 1u;
            constexpr int MS = WIDE ? kMaxMembersWide : kMaxMembers;
            unsigned long long *slot = gslots + (seq & 1u) * 2 * MS;   // [kind][member]
            // Per-lane addresses are rebuilt from the lane id on every call: kept live across the
            // whole step loop they would be spilled and reloaded on this, the latency-critical path.
            int ln = lane;
            asm volatile("" : "+v"(ln));
            post_words(slot, MS, member, ln, md, mh, ml, tag);
            unsigned touched = 0u;
            if (prefetch && ln < D / 8) {
                // candidate index travels in bits 8..31 of lo, complemented
                const int cand = min((int)(0xFFFFFFu - (ml >> 8)), last_row);
                touched = *reinterpret_cast<const volatile unsigned *>(pf_base + (size_t)cand * D + ln * 8);
            }
            const int who = ln & 31, kind = ln >> 5;
            unsigned long long g = 0ull;
            if (!WIDE) {
                good = poll_members(slot, MS, nwg, ln, tag, g);
            } else {
                // up to 128 members: a lane polls members who, who + 32, who + 64, who + 96 and keeps the largest word
                // (tag bits cleared; for the D maxima the low half is empty, so one 64-bit comparison serves both kinds)
                unsigned pending = 0u;
#pragma unroll
                for (int q = 0; q < kMaxMembersWide / 32; ++q)
                    if (who + 32 * q < nwg) pending |= 1u << q;
                unsigned spins = 0;
                while (true) {
#pragma unroll
                    for (int q = 0; q < kMaxMembersWide / 32; ++q) {
                        if (pending & (1u << q)) {
                            const unsigned long long v =
                                __hip_atomic_load(slot + kind * MS + who + 32 * q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            if ((unsigned)(v & 0xFFull) == tag) {
                                pending &= ~(1u << q);
                                const unsigned long long c = v & ~0xFFull;
                                g = c > g ? c : g;
                            }
                        }
                    }
                    if (__all(pending == 0u)) break;
                    if (++spins > kSpinLimit) {
                        good = false;
                        break;
                    }
                    if (spins > 16) __builtin_amdgcn_s_sleep(1);
                }
            }
            if (who >= nwg || !good) g = 0ull;
            const unsigned gh = (unsigned)(g >> 32), gl = (unsigned)g & 0xFFFFFF00u;
            fold_polled(gh, gl, ln, md, mh, ml);
            if (touched == 0xFFFFFFFFu && seq == 0u) good = false;   // never true: keeps the touch alive
        }
        if (lane == 0) {
            sh.rdm = md;
            sh.rhi = mh;
            sh.rlo = ml;
            if (!good) sh.abort = 1;
        }
    }
    __syncthreads();
    dm_out = sh.rdm;
    hi_out = sh.rhi;
    lo_out = sh.rlo;
    return sh.abort == 0;
}

template <int D, int RREG, int RLDS, bool WIDE>
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
    __shared__ Shared sh;

    // Workgroup ids are dealt to the 8 dies round-robin.  With a multiple of 8 heads in flight every head sits on one
    // die; with 1, 2 or 4 a head takes 8, 4 or 2 whole dies (a 32 MiB head needs the registers and LDS of two).
    int group, member;
    {
        const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
        const int dpg = a.groups <= 8 ? 8 / a.groups : 0;          // dies per head, if that divides evenly
        if ((a.groups & 7) == 0) {
            group = xcd * (a.groups >> 3) + j / a.wgpg;
            member = j % a.wgpg;
        } else if (dpg * a.groups == 8 && a.wgpg % dpg == 0) {
            group = xcd / dpg;
            member = xcd % dpg + dpg * j;
        } else {
            group = blockIdx.x / a.wgpg;
            member = blockIdx.x % a.wgpg;
        }
    }
    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = member * 4 + (tid >> 6);
    if (tid == 0) sh.abort = 0;
    __syncthreads();
    // Key blocks of 64 are dealt round-robin to the waves of the head: this lane's r-th key is
    // rowbase + rstride * r.  Neighbouring context positions tend to be neighbours in key space too, so
    // the keys a new landmark moves would otherwise pile up in one workgroup and make the others wait.
    const int rowbase = wv * 64 + lane;
    const int rstride = a.wgpg * 256;
    unsigned long long *gslots = a.slots + (size_t)group * 4 * (WIDE ? kMaxMembersWide : kMaxMembers);
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
            if (!head_max<WIDE>(mine, 0u, 0u, sh, gslots, a.wgpg, member, seq, mdm, mhi, mlo, Kh, D, a.L - 1, false)) goto bail;
            rmin = __uint_as_float(0xFFFFFFFFu - mdm);
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const bool live = rowbase + rstride * r < a.L;
            Dv[r] = live ? __builtin_inff() : -1.0f;
            ou[r] = live ? oma * (rmin / rh[r]) : ninf;
        }

        {
            int prev = 0;
            unsigned dprev = 0xFFFFFFFFu;    // bits of the D_max the last step ended with (none yet)
            for (t = 0; t < a.k; ++t) {
                unsigned lbits = 0u;
                if (t > 0) {
                    // ---- distance of every resident key to landmark `prev`
                    // The landmark row is the same for every lane: read it through the constant address
                    // space (K is never written while the kernel runs) so it arrives by scalar loads in
                    // SGPRs and serves as a broadcast operand instead of occupying VGPRs.
                    typedef const uint32_t __attribute__((address_space(4))) *cptr_t;
                    const cptr_t lp = (cptr_t)(uintptr_t)(Kh + (size_t)prev * D);
                    // its squared norm: one packed pair per lane, summed over the wave
                    // (lane l also keeps pair l mod D/2 of the landmark for the staged evaluation below)
                    const uint32_t lmw = reinterpret_cast<const uint32_t *>(Kh + (size_t)prev * D)[lane % DW];
                    const int wvl = tid >> 6;
                    // Exact evaluation widens the packed bf16 pairs on the fly.  Shift count and mask go
                    // through an empty asm so the compiler cannot treat the widened values as loop-invariant
                    // and keep a second, twice as large copy of the keys.
                    unsigned sh16 = 16u, mhi16 = 0xFFFF0000u;
                    asm volatile("" : "+s"(sh16), "+s"(mhi16));
                    // (a) Screen.  Most keys are far from the new landmark and keep their D.  With
                    // n = |k|^2, |k_i - s|^2 = n_i + n_s - 2 k_i.s, and the dot product runs on packed bf16
                    // pairs (v_dot2c_f32_bf16: two elements per instruction, a sixth of the work of
                    // widening, subtracting and squaring).  Its rounding and cancellation error is below
                    // 2^-17 (n_i + n_s); a row slot goes on to an exact evaluation unless, for every lane,
                    // the screened value exceeds D_i^2 by more than 2^-14 (n_i + n_s).  So the screen never
                    // changes a result: it only skips evaluations that cannot lower D.
                    // The packed landmark words are pinned in SGPRs for the whole step (the empty asm keeps
                    // the compiler from re-fetching them in front of every row slot).
                    uint32_t lws[DW];
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
                    unsigned needmask = 0u;          // bit r: this lane's key of row slot r may move
                    unsigned rowmask = 0u;           // bit r: some key of row slot r may move (wave-uniform)
                    float ns = 0.0f;                 // squared norm of the landmark (set once its pair has arrived)
                    uint32_t lmo = 0u;
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
                        uint4 pf[3];                 // LDS row: pieces c, c+1, c+2 in flight
                        if (MIX) {
                            pf[0] = lrows[(g * NV + 0) * 256 + tid];
                            pf[1] = lrows[(g * NV + 1) * 256 + tid];
                            __builtin_amdgcn_sched_barrier(0);
                        }
#pragma unroll
                        for (int c = 0; c < NV; ++c) {
                            if (MIX) {
                                if (c + 2 < NV) pf[(c + 2) % 3] = lrows[(g * NV + c + 2) * 256 + tid];
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
                                    const uint4 q = pf[c % 3];
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
                            lmo = (uint32_t)__shfl_xor((int)lmw, LPK);   // for the staged evaluation: the other packed word
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
                    lbits = exact_update<D, RREG, RLDS, CAP>(kr, lrows, lws, Dv, needmask, rowmask, stage_all[wvl], sres_all[wvl], tid,
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
                        if (!head_max<WIDE>(lbits, whi, wlo, sh, gslots, a.wgpg, member, seq, mdm, mhi, mlo, Kh, D, a.L - 1, true))
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

__global__ void resident_clear(unsigned long long *slots, int n, int *fail)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) slots[i] = 0ull;
    if (i == 0) *fail = 0;
}

template <int D, int RREG, int RLDS, bool WIDE = false>
hipError_t run(const ResArgs &a, hipStream_t st)
{
    hipLaunchKernelGGL((select_resident<D, RREG, RLDS, WIDE>), dim3(a.groups * a.wgpg), dim3(256), 0, st, a);
    return hipGetLastError();
}

// Key rows per lane (in registers, in LDS) of the compiled instances.
constexpr int kOpts64[][2] = {{1, 0}, {2, 0}, {4, 0}, {6, 2}};
constexpr int kOpts128[][2] = {{1, 0}, {2, 0}, {3, 1}};

// Workgroups of one instance that a compute unit holds at once, asked of the runtime for the current
// device (a host-side computation from the kernel's register and LDS use: no allocation, no launch).
// Every instance is built for two; that is the answer where there is no device to ask.
int instance_occupancy(int d, int rreg)
{
    int n = 0;
    hipError_t e = hipErrorInvalidValue;
    if (d == 64) {
        if (rreg == 1) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, select_resident<64, 1, 0, false>, 256, 0);
        else if (rreg == 2) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, select_resident<64, 2, 0, false>, 256, 0);
        else if (rreg == 4) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, select_resident<64, 4, 0, false>, 256, 0);
        else e = resident_ahead_occupancy(&n);
    } else {
        if (rreg == 1) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, select_resident<128, 1, 0, false>, 256, 0);
        else if (rreg == 2) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, select_resident<128, 2, 0, false>, 256, 0);
        else e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, select_resident<128, 3, 1, false>, 256, 0);
    }
    // (the wide instances differ from these only in the exchange's polling loop)
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return 2;
    }
    // The answer guards against a device that holds FEWER than the two the launch shapes are tuned for; where more
    // would fit (the small instances), more workgroups per head only make the exchange slower.
    return n < 2 ? n : 2;
}

}  // namespace

// Rows per lane and workgroups per head: fewest rounds over the heads, then fewest rows per lane (more
// waves per head, less serial work per step).  The workgroups of a head wait on each other, so the
// whole grid must be resident at once: groups * wgpg never exceeds compute units x workgroups per unit.
bool resident_select_shape(int H, int L, int d, const Chip &chip, ResidentShape &best)
{
    if (d != 64 && d != 128) return false;
    const int(*opts)[2] = d == 64 ? kOpts64 : kOpts128;
    const int nopts = d == 64 ? 4 : 3;
    bool found = false;
    for (int i = 0; i < nopts; ++i) {
        const int R = opts[i][0] + opts[i][1];
        const int wgpg = (L + 256 * R - 1) / (256 * R);
        // more than 32 workgroups per head only in the instance with the most rows per lane (the wide exchange)
        if (wgpg > (i == nopts - 1 ? kMaxMembersWide : kMaxMembers)) continue;
        const int occ = chip.wg_per_cu > 0 ? chip.wg_per_cu : instance_occupancy(d, opts[i][0]);
        const long long max_wg = (long long)chip.cus * occ;
        if (wgpg > max_wg) continue;                   // the group of one head could not be resident
        int groups = (int)(max_wg / wgpg);
        if (groups > kMaxResidentGroups) groups = kMaxResidentGroups;
        if (groups > H) groups = H;
        if (groups >= 8) groups -= groups % 8;         // whole groups per die
        else if (wgpg > kMaxMembers && groups == 3) groups = 2;   // whole dies per head: 1, 2 or 4 heads in flight
        else if (wgpg > kMaxMembers && groups > 4) groups = 4;
        const int rounds = (H + groups - 1) / groups;
        if (!found || rounds < best.rounds) {
            best = ResidentShape{opts[i][0], opts[i][1], wgpg, groups, rounds};
            found = true;
        }
    }
    return found;
}

size_t resident_select_workspace_bytes(int H)
{
    // the flag block, then four tagged slots per member for every head that can be in flight on any chip
    const int groups = H < kMaxResidentGroups ? H : kMaxResidentGroups;
    const int wide = H < 16 ? H : 16;        // heads in flight with more than 32 workgroups each: fewer than 16 on any chip
    return kSelectFlagBytes + round_up(((size_t)groups * 4 * kMaxMembers + (size_t)wide * 4 * kMaxMembersWide) *
                                           sizeof(unsigned long long), 256);
}

hipError_t launch_select_resident(const void *K, int H, int L, int d, const float *rho, int k, float alpha,
                                  int32_t *idx, float *score_out, void *ws, const ResidentShape &s, hipStream_t st)
{
    ResArgs a;
    a.K = reinterpret_cast<const uint16_t *>(K);
    a.rho = rho;
    a.idx = idx;
    a.score_out = score_out;
    a.fail = reinterpret_cast<int *>(ws);
    a.slots = reinterpret_cast<unsigned long long *>(reinterpret_cast<char *>(ws) + kSelectFlagBytes);
    const bool wide = s.wgpg > kMaxMembers;
    const size_t nslots = (size_t)s.groups * 4 * (wide ? kMaxMembersWide : kMaxMembers);
    a.H = H;
    a.L = L;
    a.k = k;
    a.groups = s.groups;
    a.wgpg = s.wgpg;
    a.alpha = alpha;
    hipLaunchKernelGGL(resident_clear, dim3((unsigned)((nslots + 255) / 256)), dim3(256), 0, st, a.slots, (int)nslots,
                       a.fail);
    if (wide) {
        if (s.groups > 16) return hipErrorInvalidValue;
        return d == 64 ? run<64, 6, 2, true>(a, st) : run<128, 3, 1, true>(a, st);
    }
    if (d == 64) {
        if (s.rreg == 1) return run<64, 1, 0>(a, st);
        if (s.rreg == 2) return run<64, 2, 0>(a, st);
        if (s.rreg == 4) return run<64, 4, 0>(a, st);
        // eight rows per lane: the variant that screens the expected next landmark during the exchange
        return launch_select_resident_ahead(K, H, L, rho, k, alpha, idx, score_out, a.slots, a.fail, a.groups, a.wgpg, st);
    }
    if (s.rreg == 1) return run<128, 1, 0>(a, st);
    if (s.rreg == 2) return run<128, 2, 0>(a, st);
    return run<128, 3, 1>(a, st);
}

}  // namespace ws
