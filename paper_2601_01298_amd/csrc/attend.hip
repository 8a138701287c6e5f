// N agents' decode queries attend over the k landmark rows of the synapse instead of the full
// context (Warp-Cortex Sec. 3.3 for the 1/sqrt(d_k) scale, Sec. 4 for the O(k) cost):
//     O[n,q,:] = softmax_t(scale * Q[n,q,:] . Ks[h,t,:]) . Vs[h,:,:],   h = q / (Hq/Hkv).
//
// bf16 path: a wave owns 32 query rows of one KV head and walks landmarks in tiles of 32.
// Both products are computed TRANSPOSED so that a lane always owns one query:
//     S^T = Ks_tile . Q^T     (MFMA 32x32x16: rows = landmarks, columns = queries)
//     O^T += Vs_tile^T . P^T  (rows = head dimensions, columns = queries)
// In the MFMA result layout a lane holds one column, i.e. one query, so the running maximum,
// the running denominator and the rescale factor of the online softmax are plain per-lane
// scalars; the only cross-lane traffic is one swap with lane^32, which holds the other half of
// the same column.  The probabilities leave the softmax already in the register/lane position
// the second MFMA wants for its B operand (the order of the landmarks inside the contraction
// is free, as long as Vs^T is fetched in the same order), so P never goes through LDS.  P enters
// that MFMA as a bf16 hi part plus a bf16 lo part (two instructions), which keeps 16 significant
// bits of every weight; the denominator sums the unrounded fp32 weights.
// Vs^T is built without a transpose pass: a lane fetches the 32-bit word holding head
// dimensions (2n, 2n+1) from 8 landmark rows and splits low and high halves into the operand
// of an "even dimensions" and an "odd dimensions" tile.
//
// fp32 path (small configurations): one wave per (agent, query head), plain fp32 FMAs.
//
// Both paths also exist in an indexed form that reads the chosen rows K[h, idx[h,t], :] straight from the
// cache (Sec. 3.3: the synapse holds the landmark rows only), so a caller that does not need the synapse as a
// buffer of its own skips the gather pass: same arithmetic in the same order, bit-identical output.
#include "ws_internal.h"

namespace ws {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

namespace {

__device__ __forceinline__ uint32_t bf16_rne_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

// Result layout of v_mfma_f32_32x32x*: lane l, register r hold element
// (row 8*(r/4) + 4*(l/32) + r%4, column l%32).
__device__ __forceinline__ int mfma_row(int r, int hb) { return 8 * (r >> 2) + 4 * hb + (r & 3); }

// LDS-only barrier: waits for this wave's LDS traffic, not for its global loads
__device__ __forceinline__ void lds_only_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Asynchronous 16-byte-per-lane copy global -> LDS (no registers in between): lane i of the wave reads
// base + byte_offset and lands at lds_base + 16 * i.  Completion is counted by vmcnt like any vector load;
// the compiler does not see it, so the caller waits explicitly before the barrier that publishes the data.
__device__ __forceinline__ void dma16(const void *base /* wave-uniform */, unsigned byte_offset, const void *lds_base)
{
    const unsigned la =
        __builtin_amdgcn_readfirstlane((unsigned)(size_t)(__attribute__((address_space(3))) const void *)lds_base);
    asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(byte_offset), "s"(base), "s"(la) : "memory", "m0");
}
// A 32-bit load the compiler keeps no count for (its own wait would also cover every copy in flight); the
// caller waits with wait_vmcnt and pins the first use behind that wait.
__device__ __forceinline__ void load_u32_uncounted(uint32_t &dst, const void *base /* wave-uniform */, unsigned byte_offset)
{
    asm volatile("global_load_dword %0, %1, %2" : "=v"(dst) : "v"(byte_offset), "s"(base) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// One workgroup = 4 waves = 2 query tiles of one KV head x 2 halves of the landmark range; the
// workgroups of a head are placed on the same accelerator die so its K_S/V_S rows are read from HBM
// once and from that die's L2 otherwise.  The two halves run the online softmax independently and
// are merged through LDS at the end: that gives every SIMD the same number of equally long waves
// (at 100 agents a head has 4 query tiles; without the split some SIMDs would carry two of them
// and some one).
//
// Landmark rows reach the waves through LDS.  A stage is one 32-landmark tile of each half (K and V
// rows: 4 tiles); the workgroup's 256 threads copy it global -> LDS asynchronously, 16 bytes per lane
// with no registers in between, PF stages ahead into NBUF rotating buffers, and the two query-tile
// waves of a half read the same copy.  So a workgroup fetches every landmark row once (not once per
// query tile), a wave has PF stages of memory latency covered at no cost in registers, and the
// operands arrive by LDS reads with constant offsets.  K tiles are stored with their 16-byte pieces
// XOR-swizzled by row (applied on the global side of the copy) so that the MFMA operand reads, one
// row per lane, spread over the banks; V tiles are stored as they are (their reads run along a row).
// One LDS-only barrier per stage publishes the stage and retires the buffer that is refilled next.
//
// The per-tile instruction count is what is optimised in the softmax:
//   - the score scale is folded into the exponent's FMA, the tile maximum is taken on raw scores;
//   - the running maximum is only moved when a tile exceeds it by more than 2^8, so the
//     accumulator is rescaled a few times per query instead of once per tile (weights stay below
//     2^8, harmless in fp32 and in the bf16 hi+lo split);
//   - packed conversions (v_cvt_pk_bf16_f32) and byte permutes (v_perm_b32) build the MFMA operands.
//
// IDX: Ks / Vs are the whole cache [Hkv, L, D] and landmark t of head h is row idx[h, t] (clamped into [0, L)).
// A thread then needs the index of each row it copies one step before the copy is issued: the indices of a stage
// are asked for one stage earlier than its copies (into a ring of register sets, one per stage buffer), so the copy
// never waits for the youngest load in flight.  Order of a thread's memory operations, PF = 2:
//     idx(0) idx(1) Q | copies(0) idx(2) copies(1) | idx(3) copies(2) | idx(4) copies(3) | ...
template <int D, bool IDX>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, D == 64 ? 3 : 2)))
attend_bf16(const uint16_t *__restrict__ Q, const uint16_t *__restrict__ Ks, const uint16_t *__restrict__ Vs,
            float *__restrict__ O, int N, int Hq, int Hkv, int k, float scale_log2, int parts, int splits,
            float *__restrict__ partial, const int32_t *__restrict__ idx, int L)
{
    constexpr int NK = D / 16;   // k-steps of the score product
    constexpr int NP = D / 64;   // 64-wide spans of head dimensions, each an even and an odd tile
    constexpr int CH = D / 8;    // 16-byte pieces per landmark row
    constexpr int TP = 32 * CH;  // pieces per 32-row tile
    constexpr int NLD = TP / 256;              // copies per thread and tile
    constexpr int NBUF = D == 64 ? 3 : 2;      // stage buffers (a stage: K and V tile of both halves)
    constexpr int PF = NBUF - 1;               // stages in flight ahead of the one being read
    constexpr int NC = 4 * NLD;                // copies per thread and stage
    constexpr int NI = IDX ? 2 * NLD : 0;      // index loads per thread and stage
    constexpr int NO = 2 * NP * 16;
    constexpr int STG = 4 * TP;                // pieces per stage: [half][K tile, V tile]
    constexpr int XCH = 2 * (NO + 2) * 64 * 4 / 16;                  // the merge area, in 16-byte units
    __shared__ uint4 smem[NBUF * STG > XCH ? NBUF * STG : XCH];
    // workgroup id -> (head, part): parts of one head sit on one die (ids are dealt to the 8 dies round-robin)
    // With few heads and many landmarks the landmark range is also split over `splits` workgroups (consecutive ids),
    // each leaving a normalised partial result that a second kernel merges.
    const int sp = blockIdx.x % splits, bid = blockIdx.x / splits;
    int h, part;
    if ((Hkv & 7) == 0) {
        const int xcd = bid & 7, j = bid >> 3;
        h = (j / parts) * 8 + xcd;
        part = j % parts;
    } else {
        h = bid / parts;
        part = bid % parts;
    }
    const int g = Hq / Hkv;
    const int M = N * g;         // query rows that read this KV head
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // the same for every lane: what follows from it is scalar
    const int lane = tid & 63, nq = lane & 31, hb = lane >> 5;
    const uint16_t *Kh = Ks + (size_t)h * (IDX ? L : k) * D;
    const uint16_t *Vh = Vs + (size_t)h * (IDX ? L : k) * D;
    const int wt = wave & 1, half = wave >> 1;
    const int tile = part * 2 + wt;
    const bool tile_live = tile * 32 < M;    // wave-uniform
    const int m = tile * 32 + nq;
    const bool valid = m < M;
    const int mc = valid ? m : M - 1;
    const int agent = mc / g, qh = h * g + mc % g;

    f32x16_t oacc[2 * NP];
#pragma unroll
    for (int i = 0; i < 2 * NP; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[i][r] = 0.0f;
    float mref = -__builtin_inff();   // reference maximum (log2 units) the weights are taken against
    float lrun = 0.0f;

    const int nTall = (k + 31) / 32;
    const int T0 = (int)((long long)sp * nTall / splits);             // this workgroup's tiles: [T0, nT)
    const int nT = (int)((long long)(sp + 1) * nTall / splits);
    const int tA = (nT - T0 + 1) / 2;  // half 0 walks tiles [T0, T0 + tA), half 1 [T0 + tA, nT): tA stages, the last may lack half 1

    // ---- the copy: thread `tid` moves piece q = tid + 256 i of a tile, i.e. row q / CH, LDS slot q % CH; the K tile's
    // slot c of row r holds piece c ^ (r & 7) (256 / CH rows further on the swizzle is the same: a multiple of 8).
    // Byte offsets inside a head are 32-bit (k < 2^24 rows of at most 256 bytes); a row past the end clamps to the last.
    constexpr unsigned RB = D * 2;                                   // bytes per landmark row
    const int crow = tid / CH;
    const unsigned kpiece = (unsigned)(((tid % CH) ^ (crow & 7)) * 16);
    const unsigned vpiece = (unsigned)((tid % CH) * 16);
    const unsigned last = (unsigned)(k - 1) * RB;
    unsigned off0 = (unsigned)(T0 * 32 + crow) * RB;                 // this thread's first row of the next stage, half 0 ...
    unsigned off1 = (unsigned)((T0 + tA) * 32 + crow) * RB;          // ... and half 1 (may lie past the end: clamped, never read)
    // indexed form: ring of index register sets; set s holds the rows of the stage that goes to buffer s
    uint32_t ring[NBUF][IDX ? 2 * NLD : 1];
    const int32_t *idxh = idx + (IDX ? (size_t)h * k : 0);
    int pos0 = T0 * 32 + crow, pos1 = (T0 + tA) * 32 + crow;         // landmark positions of the next index loads
    auto ask = [&](int bi) {                                         // indices of the next stage not asked for yet
        if constexpr (IDX) {
#pragma unroll
            for (int i = 0; i < NLD; ++i) {
                load_u32_uncounted(ring[bi][2 * i], idxh, 4u * (unsigned)min(pos0 + i * (256 / CH), k - 1));
                load_u32_uncounted(ring[bi][2 * i + 1], idxh, 4u * (unsigned)min(pos1 + i * (256 / CH), k - 1));
            }
            pos0 += 32;
            pos1 += 32;
        }
    };
    auto issue = [&](int bi) {                                       // bi: stage buffer, a compile-time constant at every call
        uint4 *buf = smem + bi * STG + wave * 64;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            unsigned r0, r1;
            if constexpr (IDX) {                                     // (the caller has waited for this set)
                asm volatile("" : "+v"(ring[bi][2 * i]), "+v"(ring[bi][2 * i + 1]));
                r0 = (unsigned)min(max((int)ring[bi][2 * i], 0), L - 1) * RB;
                r1 = (unsigned)min(max((int)ring[bi][2 * i + 1], 0), L - 1) * RB;
            } else {
                r0 = min(off0 + (unsigned)(i * (256 / CH)) * RB, last);
                r1 = min(off1 + (unsigned)(i * (256 / CH)) * RB, last);
            }
            dma16(Kh, r0 + kpiece, buf + 0 * TP + 256 * i);
            dma16(Vh, r0 + vpiece, buf + 1 * TP + 256 * i);
            dma16(Kh, r1 + kpiece, buf + 2 * TP + 256 * i);
            dma16(Vh, r1 + vpiece, buf + 3 * TP + 256 * i);
        }
        off0 += 32 * RB;
        off1 += 32 * RB;
    };

    // The query rows are asked for first and the first stages' copies right behind them: every workgroup starts at the
    // same moment, so what is asked for first arrives first, and the first tile needs the queries and stage 0 only.
    // The query loads are written as assembly so that the compiler keeps no count for them (its wait at their first use,
    // inside the loop, would also cover whatever copies are in flight by then); the wait below lets exactly the copies
    // stay in flight, and the empty statement behind it pins the operands' first use after that wait.
    const uint16_t *qrow = Q + ((size_t)agent * Hq + qh) * D + hb * 8;
    u32x4_t qw[NK];
    if constexpr (IDX) {
        ask(0);
        ask(1);
    }
#pragma unroll
    for (int kk = 0; kk < NK; ++kk)
        asm volatile("global_load_dwordx4 %0, %1, off offset:%2" : "=v"(qw[kk]) : "v"(qrow), "n"(kk * 32) : "memory");
    if constexpr (IDX) {
        wait_vmcnt<0>();                       // the first two stages' indices (and the queries) are in
#pragma unroll
        for (int p = 0; p < PF; ++p) {
            if (p < tA) issue(p);
            if (p + 2 <= PF) ask(p + 2);
        }
        // from here on every stage asks for one set of indices and issues one set of copies, in that order
    } else {
#pragma unroll
        for (int p = 0; p < PF; ++p)
            if (p < tA) issue(p);
        if (tA >= PF) wait_vmcnt<PF * NC>();
        else wait_vmcnt<0>();
    }
    bf16x8_t qf[NK];
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) {
        asm volatile("" : "+v"(qw[kk]));
        qf[kk] = __builtin_bit_cast(bf16x8_t, qw[kk]);
    }

    // LDS read positions of this lane: K row nq of the tile (its swizzled pieces), V words of head dimensions 2nq, 2nq+1
    int kslot[NK];
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) kslot[kk] = nq * CH + ((2 * kk + hb) ^ (nq & 7));

    // One stage: `bi` is its buffer (a constant at every call, so LDS offsets are immediates)
    auto stage = [&](int sidx, int bi) {
        // this wave's copies of the stage have landed (those of later stages may still be in flight) ...
        // (younger than them: the next stage's copies and, indexed, the index loads behind which they were issued)
        if (PF == 2 && sidx + 1 < tA) wait_vmcnt<NC + NI>();
        else wait_vmcnt<0>();
        // ... and so have everybody's; all waves are through with the buffer that is refilled next
        lds_only_barrier();
        if constexpr (IDX) ask(bi);            // rows of stage sidx + PF + 1; its set last served stage sidx
        if (sidx + PF < tA) {
            // indexed: the set of stage sidx + PF, asked for one stage ago, has only the previous stage's copies and
            // the loads just issued behind it
            if constexpr (IDX) wait_vmcnt<NC + NI>();
            issue((bi + PF) % NBUF);
        }
        const int t = T0 + (half ? tA + sidx : sidx);
        if (!tile_live || t >= nT) return;             // wave-uniform
        const int t0 = t * 32;
        const uint4 *sK = smem + bi * STG + (half * 2 + 0) * TP;
        const uint32_t *sV = reinterpret_cast<const uint32_t *>(smem + bi * STG + (half * 2 + 1) * TP);

        bf16x8_t kf[NK];
#pragma unroll
        for (int kk = 0; kk < NK; ++kk) kf[kk] = __builtin_bit_cast(bf16x8_t, sK[kslot[kk]]);
        // V: the 32-bit word holding head dimensions (2 nq, 2 nq + 1) of 16 landmark rows; contraction slot
        // (kk2, hb, e) <-> landmark t0 + mfma_row(8*kk2+e, hb) = t0 + 16 kk2 + 8 (e/4) + 4 hb + e%4.
        uint32_t vd[2][NP][8];
#pragma unroll
        for (int kk2 = 0; kk2 < 2; ++kk2)
#pragma unroll
            for (int e = 0; e < 8; ++e)
#pragma unroll
                for (int p = 0; p < NP; ++p)
                    vd[kk2][p][e] = sV[(16 * kk2 + 8 * (e >> 2) + 4 * hb + (e & 3)) * (D / 2) + 32 * p + nq];

        // ---- S^T tile: rows = landmarks t0..t0+31, columns = queries
        f32x16_t sacc;
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[r] = 0.0f;
#pragma unroll
        for (int kk = 0; kk < NK; ++kk) sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], qf[kk], sacc, 0, 0, 0);
        if (t0 + 32 > k) {       // ragged last tile: landmarks past k get zero weight
            asm volatile("" ::: "memory");              // (keeps this a branch: as selects it would run on every tile)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (t0 + mfma_row(r, hb) >= k) sacc[r] = -__builtin_inff();
        }

        // ---- online softmax, one query per lane (its other 16 landmarks sit in lane^32)
        float tmax = sacc[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) tmax = fmaxf(tmax, sacc[r]);
        tmax *= scale_log2;
        if (__any(tmax > mref + 8.0f)) {
            // some query of this wave moved: take the exact maximum over both half-columns and rescale
            const float tm = fmaxf(tmax, __shfl_xor(tmax, 32));
            const float mnew = fmaxf(mref, tm);
            const float corr = __builtin_amdgcn_exp2f(mref - mnew);     // 0 on the first tile
            mref = mnew;
            lrun *= corr;
#pragma unroll
            for (int i = 0; i < 2 * NP; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[i][r] *= corr;
        }
        // probabilities as bf16 hi + bf16 lo (16 significant bits): one bf16 alone would cost up to
        // 2^-9 relative error per weight, which is the whole error budget of the output
        uint32_t pkh[8], pkl[8];
        // (-1, 0) and (0, -1) as bf16 pairs, kept in registers: written as an immediate operand the first one is
        // encoded as the inline constant -1.0, which this instruction reads as the fp32 pattern, i.e. as (0, -1)
        uint32_t c10 = 0x0000BF80u, c01 = 0xBF800000u;
        asm volatile("" : "+v"(c10), "+v"(c01));
        const bf16x2_t kMinusOneZero = __builtin_bit_cast(bf16x2_t, c10);
        const bf16x2_t kZeroMinusOne = __builtin_bit_cast(bf16x2_t, c01);
        float psum = 0.0f;
        const float nmref = -mref;
#pragma unroll
        for (int w = 0; w < 8; ++w) {
            f32x2_t pv;
            pv[0] = __builtin_amdgcn_exp2f(fmaf(sacc[2 * w], scale_log2, nmref));
            pv[1] = __builtin_amdgcn_exp2f(fmaf(sacc[2 * w + 1], scale_log2, nmref));
            psum += pv[0] + pv[1];
            const bf16x2_t hi2 = __builtin_convertvector(pv, bf16x2_t);
            // what the bf16 pair leaves of each weight, straight from the packed pair: p - hi.x * 1 - hi.y * 0 in one
            // dot-product instruction (exact: the difference has at most 16 significant bits)
            f32x2_t rest;
            rest[0] = __builtin_amdgcn_fdot2_f32_bf16(hi2, kMinusOneZero, pv[0], false);
            rest[1] = __builtin_amdgcn_fdot2_f32_bf16(hi2, kZeroMinusOne, pv[1], false);
            pkh[w] = __builtin_bit_cast(uint32_t, hi2);
            pkl[w] = __builtin_bit_cast(uint32_t, __builtin_convertvector(rest, bf16x2_t));
        }
        lrun += psum;

        // ---- O^T += Vs^T . P^T
#pragma unroll
        for (int kk2 = 0; kk2 < 2; ++kk2) {
            const bf16x8_t pfh = __builtin_bit_cast(
                bf16x8_t, make_uint4(pkh[4 * kk2], pkh[4 * kk2 + 1], pkh[4 * kk2 + 2], pkh[4 * kk2 + 3]));
            const bf16x8_t pfl = __builtin_bit_cast(
                bf16x8_t, make_uint4(pkl[4 * kk2], pkl[4 * kk2 + 1], pkl[4 * kk2 + 2], pkl[4 * kk2 + 3]));
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                uint32_t ev[4], od[4];
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    // low halves (even head dimension) and high halves (odd) of two landmark rows
                    ev[w] = __builtin_amdgcn_perm(vd[kk2][p][2 * w + 1], vd[kk2][p][2 * w], 0x05040100u);
                    od[w] = __builtin_amdgcn_perm(vd[kk2][p][2 * w + 1], vd[kk2][p][2 * w], 0x07060302u);
                }
                const bf16x8_t ve = __builtin_bit_cast(bf16x8_t, make_uint4(ev[0], ev[1], ev[2], ev[3]));
                const bf16x8_t vo = __builtin_bit_cast(bf16x8_t, make_uint4(od[0], od[1], od[2], od[3]));
                oacc[2 * p] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ve, pfh, oacc[2 * p], 0, 0, 0);
                oacc[2 * p] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ve, pfl, oacc[2 * p], 0, 0, 0);
                oacc[2 * p + 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vo, pfh, oacc[2 * p + 1], 0, 0, 0);
                oacc[2 * p + 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vo, pfl, oacc[2 * p + 1], 0, 0, 0);
            }
        }
    };
    for (int s0 = 0; s0 < tA; s0 += NBUF) {
#pragma unroll
        for (int bi = 0; bi < NBUF; ++bi)
            if (s0 + bi < tA) stage(s0 + bi, bi);
    }

    // ---- merge the two halves of the landmark range: half 1 hands its state to half 0 through LDS
    // (the merge area lies over the stage buffers: every wave is through with them first)
    __syncthreads();
    float(*xch)[NO + 2][64] = reinterpret_cast<float(*)[NO + 2][64]>(smem);
    if (half == 1) {
        xch[wt][NO][lane] = mref;
        xch[wt][NO + 1][lane] = lrun;
#pragma unroll
        for (int i = 0; i < 2 * NP; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) xch[wt][i * 16 + r][lane] = oacc[i][r];
    }
    __syncthreads();
    if (half == 0 && tile_live) {
        const float m1 = xch[wt][NO][lane], l1 = xch[wt][NO + 1][lane];
        const float mm = fmaxf(mref, m1);                 // finite: half 0 always holds landmark 0
        const float f0 = __builtin_amdgcn_exp2f(mref - mm), f1 = __builtin_amdgcn_exp2f(m1 - mm);
        float l = lrun * f0 + l1 * f1;
        l += __shfl_xor(l, 32);
        const float inv = 1.0f / l;
        const float g0 = f0 * inv, g1 = f1 * inv;
#pragma unroll
        for (int i = 0; i < 2 * NP; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[i][r] = oacc[i][r] * g0 + xch[wt][i * 16 + r][lane] * g1;
        if (valid) {
            // one workgroup per landmark range: the result; several: a partial row [D values, maximum, denominator, pad]
            const size_t rowid = (size_t)agent * Hq + qh;
            float *orow = splits == 1 ? O + rowid * D : partial + ((size_t)sp * N * Hq + rowid) * (D + 4);
#pragma unroll
            for (int p = 0; p < NP; ++p)
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    // registers 4b..4b+3 of the even and odd tile interleave into 8 consecutive dims
                    float *dst = orow + 64 * p + 16 * b + 8 * hb;
                    *reinterpret_cast<float4 *>(dst) = make_float4(oacc[2 * p][4 * b], oacc[2 * p + 1][4 * b],
                                                                   oacc[2 * p][4 * b + 1], oacc[2 * p + 1][4 * b + 1]);
                    *reinterpret_cast<float4 *>(dst + 4) = make_float4(oacc[2 * p][4 * b + 2], oacc[2 * p + 1][4 * b + 2],
                                                                       oacc[2 * p][4 * b + 3], oacc[2 * p + 1][4 * b + 3]);
                }
            if (splits > 1 && hb == 0) *reinterpret_cast<float2 *>(orow + D) = make_float2(mm, l);
        }
    }
}

// Merge of the partial rows of a split landmark range: O = sum_s w_s O_s / sum_s w_s, w_s = l_s 2^(m_s - max m).
template <int D>
__global__ void __launch_bounds__(256)
attend_merge(const float *__restrict__ partial, float *__restrict__ O, long long rows, int splits)
{
    constexpr int TPR = D / 4;                     // threads per row, a float4 each
    const long long row = (long long)blockIdx.x * (256 / TPR) + threadIdx.x / TPR;
    const int c = threadIdx.x % TPR;
    if (row >= rows) return;
    float mmax = -__builtin_inff();
    for (int s = 0; s < splits; ++s) mmax = fmaxf(mmax, partial[((size_t)s * rows + row) * (D + 4) + D]);
    float4 acc = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    float wsum = 0.0f;
    for (int s = 0; s < splits; ++s) {
        const float *pr = partial + ((size_t)s * rows + row) * (D + 4);
        const float w = pr[D + 1] * __builtin_amdgcn_exp2f(pr[D] - mmax);
        const float4 v = *reinterpret_cast<const float4 *>(pr + 4 * c);
        acc.x = fmaf(w, v.x, acc.x);
        acc.y = fmaf(w, v.y, acc.y);
        acc.z = fmaf(w, v.z, acc.z);
        acc.w = fmaf(w, v.w, acc.w);
        wsum += w;
    }
    const float inv = 1.0f / wsum;
    *reinterpret_cast<float4 *>(O + row * D + 4 * c) = make_float4(acc.x * inv, acc.y * inv, acc.z * inv, acc.w * inv);
}

template <int D, bool IDX>
__global__ void __launch_bounds__(64)
attend_f32(const float *__restrict__ Q, const float *__restrict__ Ks, const float *__restrict__ Vs,
           float *__restrict__ O, int Hq, int Hkv, int k, float scale, const int32_t *__restrict__ idx, int L)
{
    constexpr int NC = D / 64;   // output dims per lane
    __shared__ float ps[64];
    __shared__ int rs[64];       // cache row of each landmark of the chunk
    __shared__ float qs[D];
    const int lane = threadIdx.x;
    const int nq = blockIdx.x;             // agent * Hq + query head
    const int q = nq % Hq;
    const int h = q / (Hq / Hkv);
    const float *qrow = Q + (size_t)nq * D;
    const float *Kh = Ks + (size_t)h * (IDX ? L : k) * D;
    const float *Vh = Vs + (size_t)h * (IDX ? L : k) * D;
#pragma unroll
    for (int c = 0; c < NC; ++c) qs[lane + 64 * c] = qrow[lane + 64 * c];
    __syncthreads();

    float oacc[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) oacc[c] = 0.0f;
    float mrun = -__builtin_inff(), lrun = 0.0f;

    for (int c0 = 0; c0 < k; c0 += 64) {
        const int t = c0 + lane;
        float z = -__builtin_inff();
        int row = t;
        if (IDX && t < k) row = min(max(idx[(size_t)h * k + t], 0), L - 1);
        if (t < k) {
            const float *kr = Kh + (size_t)row * D;
            float s = 0.0f;
#pragma unroll 8
            for (int c = 0; c < D; ++c) s = fmaf(qs[c], kr[c], s);
            z = s * scale;
        }
        float cmax = z;
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) cmax = fmaxf(cmax, __shfl_xor(cmax, o));
        const float mnew = fmaxf(mrun, cmax);
        const float corr = expf(mrun - mnew);
        mrun = mnew;
        const float p = (t < k) ? expf(z - mnew) : 0.0f;
        __syncthreads();                   // previous chunk's readers are done with ps
        ps[lane] = p;
        rs[lane] = row;
        float psum = p;
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) psum += __shfl_xor(psum, o);
        lrun = lrun * corr + psum;
        __syncthreads();
        const int cnt = min(64, k - c0);
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            float acc = oacc[c] * corr;
            for (int j = 0; j < cnt; ++j) acc = fmaf(ps[j], Vh[(size_t)rs[j] * D + lane + 64 * c], acc);
            oacc[c] = acc;
        }
    }
#pragma unroll
    for (int c = 0; c < NC; ++c) O[(size_t)nq * D + lane + 64 * c] = oacc[c] / lrun;
}

}  // namespace

// Landmark-range splits for a launch: with enough (head, query tile pair) workgroups to fill the chip, one; otherwise as
// many as bring the grid to about 512 workgroups, each split keeping at least four landmark tiles.  The choice depends
// on the sizes only, so the result (the merge order) is the same on every device.
static int attend_splits(long long wgs, int k)
{
    const int nT = (k + 31) / 32;
    if (wgs >= 384 || nT < 8) return 1;
    long long s = (512 + wgs - 1) / wgs;
    if (s > nT / 4) s = nT / 4;
    if (s > 16) s = 16;
    return s < 1 ? 1 : (int)s;
}

size_t attend_workspace_bytes(bool bf16, int N, int Hq, int Hkv, int k, int d)
{
    if (!bf16 || Hkv < 1 || Hq % Hkv != 0) return 0;
    const long long M = (long long)N * (Hq / Hkv);
    const int s = attend_splits((M + 63) / 64 * Hkv, k);
    return s == 1 ? 0 : round_up((size_t)s * N * Hq * (d + 4) * sizeof(float), 256);
}

template <bool IDX>
static hipError_t launch_attend_any(const void *Q, const void *Ks, const void *Vs, const int32_t *idx, int L, bool bf16,
                                    int N, int Hq, int Hkv, int k, int d, float scale, float *O, void *ws, hipStream_t st)
{
    if (bf16) {
        const int g = Hq / Hkv;
        const long long M = (long long)N * g;
        const long long parts = (M + 63) / 64;                 // workgroups (2 query tiles each) per head
        const int splits = attend_splits(parts * Hkv, k);
        const long long blocks = parts * Hkv * splits;
        if (blocks > 0x7FFFFFFFLL) return hipErrorInvalidValue;
        const dim3 grid((unsigned)blocks);
        const float sl2 = scale * 1.4426950408889634f;
        const uint16_t *q = reinterpret_cast<const uint16_t *>(Q);
        const uint16_t *ks = reinterpret_cast<const uint16_t *>(Ks);
        const uint16_t *vs = reinterpret_cast<const uint16_t *>(Vs);
        float *part = reinterpret_cast<float *>(ws);
        const long long rows = (long long)N * Hq;
        if (d == 64) {
            hipLaunchKernelGGL((attend_bf16<64, IDX>), grid, dim3(256), 0, st, q, ks, vs, O, N, Hq, Hkv, k, sl2, (int)parts,
                               splits, part, idx, L);
            if (splits > 1)
                hipLaunchKernelGGL(attend_merge<64>, dim3((unsigned)((rows + 15) / 16)), dim3(256), 0, st, part, O, rows,
                                   splits);
        } else if (d == 128) {
            hipLaunchKernelGGL((attend_bf16<128, IDX>), grid, dim3(256), 0, st, q, ks, vs, O, N, Hq, Hkv, k, sl2, (int)parts,
                               splits, part, idx, L);
            if (splits > 1)
                hipLaunchKernelGGL(attend_merge<128>, dim3((unsigned)((rows + 7) / 8)), dim3(256), 0, st, part, O, rows,
                                   splits);
        } else {
            return hipErrorInvalidValue;
        }
    } else {
        const long long blocks = (long long)N * Hq;
        if (blocks > 0x7FFFFFFFLL) return hipErrorInvalidValue;
        const float *q = reinterpret_cast<const float *>(Q);
        const float *ks = reinterpret_cast<const float *>(Ks);
        const float *vs = reinterpret_cast<const float *>(Vs);
        if (d == 64)
            hipLaunchKernelGGL((attend_f32<64, IDX>), dim3((unsigned)blocks), dim3(64), 0, st, q, ks, vs, O, Hq, Hkv, k, scale,
                               idx, L);
        else if (d == 128)
            hipLaunchKernelGGL((attend_f32<128, IDX>), dim3((unsigned)blocks), dim3(64), 0, st, q, ks, vs, O, Hq, Hkv, k, scale,
                               idx, L);
        else
            return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_attend(const void *Q, const void *Ks, const void *Vs, bool bf16, int N, int Hq, int Hkv, int k,
                         int d, float scale, float *O, void *ws, hipStream_t st)
{
    return launch_attend_any<false>(Q, Ks, Vs, nullptr, 0, bf16, N, Hq, Hkv, k, d, scale, O, ws, st);
}

hipError_t launch_attend_indexed(const void *Q, const void *K, const void *V, const int32_t *idx, bool bf16, int N,
                                 int Hq, int Hkv, int L, int k, int d, float scale, float *O, void *ws, hipStream_t st)
{
    return launch_attend_any<true>(Q, K, V, idx, L, bf16, N, Hq, Hkv, k, d, scale, O, ws, st);
}

}  // namespace ws
