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
// Vs^T needs no transpose pass and no vector instruction: the LDS transpose read
// (ds_read_b64_tr_b16) hands a lane the values of ONE head dimension from four consecutive
// landmark rows, which is the operand layout of the second MFMA.
//
// fp32 path (small configurations): one wave per (agent, query head), plain fp32 FMAs.
//
// Both paths also exist in an indexed form that reads the chosen rows K[h, idx[h,t], :] straight from the
// cache (Sec. 3.3: the synapse holds the landmark rows only), so a caller that does not need the synapse as a
// buffer of its own skips the gather pass: same arithmetic in the same order, bit-identical output.
#include <type_traits>

#include "ws_internal.h"

namespace ws {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

namespace {

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
// row per lane, spread over the banks; V tiles likewise, by the rule their transpose reads need (see read_v).
// One LDS-only barrier per stage publishes the stage and retires the buffer that is refilled next.
//
// The per-tile instruction count is what is optimised in the softmax:
//   - the score scale is folded into the exponent's FMA, the tile maximum is taken on raw scores;
//   - the running maximum is only moved when a tile exceeds it by more than 2^8, so the
//     accumulator is rescaled a few times per query instead of once per tile (weights stay below
//     2^8, harmless in fp32 and in the bf16 hi+lo split);
//   - packed conversions (v_cvt_pk_bf16_f32) build the weights' operand, the V operand comes ready from the LDS.
//
// IDX: Ks / Vs are the whole cache [Hkv, L, D] and landmark t of head h is row idx[h, t] (clamped into [0, L)).
// A thread then needs the index of each row it copies one step before the copy is issued: the indices of a stage
// are asked for one stage earlier than its copies (into a ring of register sets, one per stage buffer), so the copy
// never waits for the youngest load in flight.  Order of a thread's memory operations (one stage ahead):
//     idx(0) idx(1) Q | copies(0) | idx(2) copies(1) | idx(3) copies(2) | ...
template <int D, bool IDX>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(D == 64 ? 3 : 2, D == 64 ? 3 : 2)))
attend_bf16(const uint16_t *__restrict__ Q, const uint16_t *__restrict__ Ks, const uint16_t *__restrict__ Vs,
            float *__restrict__ O, int N, int Hq, int Hkv, int k, float scale_log2, int parts, int splits,
            float *__restrict__ partial, const int32_t *__restrict__ idx, int L)
{
    constexpr int NK = D / 16;   // k-steps of the score product
    constexpr int NP = D / 64;   // 64-wide spans of head dimensions, each two output tiles of 32 dimensions
    constexpr int CH = D / 8;    // 16-byte pieces per landmark row
    constexpr int TP = 32 * CH;  // pieces per 32-row tile
    constexpr int NLD = TP / 256;              // copies per thread and tile
    constexpr int NBUF = 2;                    // stage buffers (a stage: K and V tile of both halves); a third one, i.e. two
                                               // stages in flight, is no faster at either head dimension (the loop does not wait for memory)
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
    // Which wave pair takes which half alternates from one group of 256 workgroups to the next (a compute unit's three
    // workgroups come from three such groups): an odd tile count gives half 0 one tile more, and that tile should not
    // land on the same two SIMDs three times.
    const int wt = wave & 1, half = (wave >> 1) ^ (((blockIdx.x / splits) >> 8) & 1);
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
    // V: slot c of row r holds piece c ^ vswz(r), vswz(r) = 4 ((r >> 1) & 1) at d = 64, 4 (r & 3) at d = 128 (a function
    // of r & 7, so it is the same for every row a thread copies)
    const unsigned vpiece = (unsigned)(((tid % CH) ^ (D == 64 ? ((crow >> 1) & 1) << 2 : (crow & 3) << 2)) * 16);
    const unsigned last = (unsigned)(k - 1) * RB;
    unsigned off0 = (unsigned)(T0 * 32 + crow) * RB;                 // this thread's first V row of the next stage, half 0;
    const unsigned hoff = (unsigned)(tA * 32) * RB;                  // half 1 lies this much further on (uniform; past the end: clamped, never read)
    // indexed form: ring of index register sets; set s holds the rows of the stage that goes to buffer s
    // (half 0, half 1 per copy pass)
    uint32_t ring[NBUF][IDX ? 2 * NLD : 1];
    const int32_t *idxh = idx + (IDX ? (size_t)h * k : 0);
    int pos0 = T0 * 32 + crow;                                       // landmark position of the next index loads, half 0
    auto ask = [&](int bi) {                                         // indices of the next stage not asked for yet
        if constexpr (IDX) {
#pragma unroll
            for (int i = 0; i < NLD; ++i) {
                const int a0 = pos0 + i * (256 / CH), a1 = a0 + tA * 32;
                load_u32_uncounted(ring[bi][2 * i + 0], idxh, 4u * (unsigned)min(a0, k - 1));
                load_u32_uncounted(ring[bi][2 * i + 1], idxh, 4u * (unsigned)min(a1, k - 1));
            }
            pos0 += 32;
        }
    };
    auto row_of = [&](uint32_t &reg) {                               // (the caller has waited for this register's load)
        asm volatile("" : "+v"(reg));
        return (unsigned)min(max((int)reg, 0), L - 1) * RB;
    };
    auto issue = [&](int bi) {                                       // bi: stage buffer, a compile-time constant at every call
        uint4 *buf = smem + bi * STG + wave * 64;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            unsigned r0, r1;
            if constexpr (IDX) {
                r0 = row_of(ring[bi][2 * i + 0]);
                r1 = row_of(ring[bi][2 * i + 1]);
            } else {
                r0 = min(off0 + (unsigned)(i * (256 / CH)) * RB, last);
                r1 = min(off0 + hoff + (unsigned)(i * (256 / CH)) * RB, last);
            }
            dma16(Kh, r0 + kpiece, buf + 0 * TP + 256 * i);
            dma16(Vh, r0 + vpiece, buf + 1 * TP + 256 * i);
            dma16(Kh, r1 + kpiece, buf + 2 * TP + 256 * i);
            dma16(Vh, r1 + vpiece, buf + 3 * TP + 256 * i);
        }
        off0 += 32 * RB;
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
    if constexpr (IDX) wait_vmcnt<0>();        // the first two stages' indices (and the queries) are in
    // (indexed: from here on every stage asks for one set of indices and issues one set of copies, in that order)
#pragma unroll
    for (int p = 0; p < PF; ++p) {
        if (p < tA) issue(p);
        if (IDX && p + 2 <= PF) ask(p + 2);
    }
    // The queries are in.  With one stage ahead the first stage waits for its copies next anyway, so everything is
    // waited for, on every path; with more stages ahead the later ones stay in flight.
    if (PF > 1 && tA >= PF) wait_vmcnt<PF * NC + (PF - 1) * NI>();
    else wait_vmcnt<0>();
    bf16x8_t qf[NK];
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) {
        asm volatile("" : "+v"(qw[kk]));
        qf[kk] = __builtin_bit_cast(bf16x8_t, qw[kk]);
    }

    // ---- the tile loop: scores, softmax weights and P.V of a tile one after the other.  (Interleaving the matrix
    // instructions of neighbouring tiles with the vector work inside a wave, as the density sweep does, was built and
    // measured: 25.1 us against 23.7 - three waves per SIMD already cover each other's matrix phases, and the
    // interleaved form needs 15 to 37 more vector instructions per tile.)
    const int n = !tile_live ? 0 : (half ? max(nT - T0 - tA, 0) : tA);     // this wave's tiles (wave-uniform)
    const int tbase = T0 + (half ? tA : 0);
    constexpr int NA = 4 * NP;                 // matrix instructions of half a tile's P.V

    f32x16_t sacc;                             // scores of the tile whose weights are formed next
    uint32_t pkh[8], pkl[8];                   // weights, bf16 hi and lo
    uint32_t vt[2][2 * NP][4];                 // V^T operands: [landmark half][32 head dimensions][8 landmarks of this lane's dimension]

    // (-1, 0) and (0, -1) as bf16 pairs, kept in (scalar) registers: written as an immediate operand the first one is
    // encoded as the inline constant -1.0, which this instruction reads as the fp32 pattern, i.e. as (0, -1)
    uint32_t c10 = 0x0000BF80u, c01 = 0xBF800000u;
    asm volatile("" : "+s"(c10), "+s"(c01));
    const bf16x2_t kMinusOneZero = __builtin_bit_cast(bf16x2_t, c10);
    const bf16x2_t kZeroMinusOne = __builtin_bit_cast(bf16x2_t, c01);

    // weights of landmark pair w (score registers 2w, 2w + 1) as bf16 hi + bf16 lo (16 significant bits): one bf16 alone
    // would cost up to 2^-9 relative error per weight, which is the whole error budget of the output
    auto weights = [&](int w) {
        f32x2_t pv;
        pv[0] = __builtin_amdgcn_exp2f(fmaf(sacc[2 * w], scale_log2, -mref));
        pv[1] = __builtin_amdgcn_exp2f(fmaf(sacc[2 * w + 1], scale_log2, -mref));
        lrun += pv[0] + pv[1];
        const bf16x2_t hi2 = __builtin_convertvector(pv, bf16x2_t);
        // what the bf16 pair leaves of each weight, straight from the packed pair: p - hi.x * 1 - hi.y * 0 in one
        // dot-product instruction (exact: the difference has at most 16 significant bits)
        f32x2_t rest;
        rest[0] = __builtin_amdgcn_fdot2_f32_bf16(hi2, kMinusOneZero, pv[0], false);
        rest[1] = __builtin_amdgcn_fdot2_f32_bf16(hi2, kZeroMinusOne, pv[1], false);
        pkh[w] = __builtin_bit_cast(uint32_t, hi2);
        pkl[w] = __builtin_bit_cast(uint32_t, __builtin_convertvector(rest, bf16x2_t));
    };
    // matrix instruction i of landmark half kk2 of a tile's P.V: hi parts of every output tile first, then lo parts
    auto pv_mfma = [&](int i, int kk2) {
        const int lo = i / (2 * NP), p = i % (2 * NP);
        const uint32_t *pk = lo ? pkl : pkh;
        const bf16x8_t pf = __builtin_bit_cast(
            bf16x8_t, make_uint4(pk[4 * kk2], pk[4 * kk2 + 1], pk[4 * kk2 + 2], pk[4 * kk2 + 3]));
        const uint32_t *v = vt[kk2][p];
        const bf16x8_t vf = __builtin_bit_cast(bf16x8_t, make_uint4(v[0], v[1], v[2], v[3]));
        oacc[p] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, oacc[p], 0, 0, 0);
    };
    // K operand kk of the tile in the K slot of buffer `bi`: row nq, piece (2 kk + hb) ^ (nq & 7).  The row starts at a
    // multiple of 16 CH bytes, so the swizzle is an XOR of the byte address with 32 kk: one address register, not NK.
    // (this half's K slot is part of the lane's address, so that the buffer is an immediate offset)
    const unsigned kaddr = ((unsigned)(nq * CH * 16) | (unsigned)(((nq & 7) ^ hb) * 16)) + (unsigned)(half * 2 * TP * 16);
    auto read_k = [&](int bi, int kk) {
        const char *sK = reinterpret_cast<const char *>(smem + bi * STG);
        return __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4 *>(sK + (kaddr ^ (unsigned)(32 * kk))));
    };
    // V^T operands of landmark half kk2 of the stage in buffer `bi`.  Contraction slot (kk2, hb, e) stands for landmark
    // mfma_row(8 kk2 + e, hb) = 16 kk2 + 8 (e / 4) + 4 hb + e % 4 of the tile (the weights' registers fix that), i.e. a
    // lane's 8 slots are two runs of 4 consecutive landmarks, and it needs them for ONE head dimension (32 p + nq).
    // The transpose read works on blocks of 16 lanes: lane j of a block fetches 8 bytes, and lane i receives element
    // i % 4 of the pieces fetched by lanes i / 4, 4 + i / 4, 8 + i / 4, 12 + i / 4.  So lanes 4 e .. 4 e + 3 of a block
    // fetch 16 consecutive head dimensions of landmark e of the run, and lane i comes away with dimension i of all
    // four.  Blocks 0, 1 serve dimensions 0-15, 16-31 at hb = 0, blocks 2, 3 at hb = 1.  Rows of a run lie 2 D bytes
    // apart, which would put them on the same banks: pieces are stored XOR-swizzled by row (see the copy above).  The
    // swizzle depends on the row modulo 8 only, i.e. on the lane and not on the run, but it moves whole 32-dimension
    // spans: one base address per span, the run an immediate offset.
    const int vrow = 4 * hb + (lane & 15) / 4;                               // the row this lane fetches, counted from the run's base 16 kk2 + 8 eh
    const int vdim = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);               // first of the 4 dimensions this lane fetches
    const unsigned vswz = D == 64 ? ((vrow >> 1) & 1) << 2 : (vrow & 3) << 2;
    unsigned vaddr[2 * NP];
#pragma unroll
    for (int p = 0; p < 2 * NP; ++p)
        vaddr[p] = (unsigned)((half * 2 + 1) * TP * 16 + vrow * (int)RB) +
                   ((((unsigned)(32 * p + vdim) >> 3) ^ vswz) * 16 + (vdim & 4) * 2);
    auto read_v = [&](int bi, int kk2) {
        typedef __attribute__((address_space(3))) s16x4_t *lds_s16x4;
        const char *sV = reinterpret_cast<const char *>(smem + bi * STG);
#pragma unroll
        for (int p = 0; p < 2 * NP; ++p)
#pragma unroll
            for (int eh = 0; eh < 2; ++eh) {
                const s16x4_t v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(sV + vaddr[p] + (16 * kk2 + 8 * eh) * RB));
                vt[kk2][p][2 * eh] = (uint32_t)(uint16_t)v[0] | ((uint32_t)(uint16_t)v[1] << 16);
                vt[kk2][p][2 * eh + 1] = (uint32_t)(uint16_t)v[2] | ((uint32_t)(uint16_t)v[3] << 16);
            }
    };
    // maximum of score registers [r0, r1) of `sc`, folded into tm
    auto fold_max = [&](const f32x16_t &sc, float tm, int r0, int r1) {
#pragma unroll
        for (int r = r0; r < r1; ++r) tm = fmaxf(tm, sc[r]);
        return tm;
    };
    // The scores in `sacc` are those of tile j (rows = landmarks, columns = queries), tm their maximum per lane: mask a
    // ragged last tile, then move the reference maximum if some query of this wave exceeds it by more than 2^8.
    auto settle = [&](int j, float tm) {
        const int t0 = (tbase + j) * 32;
        if (t0 + 32 > k) {       // ragged last tile: landmarks past k get zero weight
            const int hbm = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u)) >> 5;
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (t0 + mfma_row(r, hbm) >= k) sacc[r] = -__builtin_inff();
            tm = fold_max(sacc, -__builtin_inff(), 0, 16);
        }
        float tmax = tm * scale_log2;
        if (__any(tmax > mref + 8.0f)) {
            // take the exact maximum over both half-columns (lane ^ 32 holds the other 16 landmarks) and rescale
            const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(tmax), __float_as_uint(tmax), false, false);
            const float mnew = fmaxf(mref, fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1])));
            const float corr = __builtin_amdgcn_exp2f(mref - mnew);     // 0 on the first tile
            mref = mnew;
            lrun *= corr;
#pragma unroll
            for (int i = 0; i < 2 * NP; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[i][r] *= corr;
        }
    };
    auto scores_of = [&](int bi) {             // the tile in the K slot of buffer `bi` -> sacc, plain order
        bf16x8_t kf[NK];
#pragma unroll
        for (int kk = 0; kk < NK; ++kk) kf[kk] = read_k(bi, kk);
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[r] = 0.0f;
#pragma unroll
        for (int kk = 0; kk < NK; ++kk) sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], qf[kk], sacc, 0, 0, 0);
    };

    // One stage: `bi` is its buffer (a constant at every call, so LDS offsets are immediates)
    auto stage = [&](int sidx, int bi, auto tail) {   // tail: the stage after the last whole round, nothing follows it
        // this wave's copies of the stage have landed (those of later stages may still be in flight) ...
        // (younger than them: the next stage's copies and, indexed, the index loads behind which they were issued)
        if (PF == 2 && sidx + 1 < tA) wait_vmcnt<NC + NI>();
        else wait_vmcnt<0>();
        // ... and so have everybody's; all waves are through with the buffer that is refilled next
        lds_only_barrier();
        // rows of stage sidx + PF + 1; its set last served stage sidx.  Asked for only if that stage exists: a load
        // whose result nobody reads has a destination the compiler counts as free while the load is still in flight.
        if constexpr (IDX && !decltype(tail)::value) {
            if (sidx + PF + 1 < tA) ask(bi);
        }
        if (!decltype(tail)::value && sidx + PF < tA) {
            // indexed: the set of stage sidx + PF, asked for one stage ago, has only the previous stage's copies and
            // the loads just issued behind it
            if constexpr (IDX) wait_vmcnt<NC + NI>();
            issue((bi + PF) % NBUF);
        }
        if (sidx < n) {
            read_v(bi, 0);
            read_v(bi, 1);
            scores_of(bi);
            settle(sidx, fold_max(sacc, -__builtin_inff(), 0, 16));
#pragma unroll
            for (int w = 0; w < 8; ++w) weights(w);
#pragma unroll
            for (int i = 0; i < NA; ++i) pv_mfma(i, 0);
#pragma unroll
            for (int i = 0; i < NA; ++i) pv_mfma(i, 1);
        }
    };
    // Whole rounds of the buffer ring first, every stage of a round unconditionally, then the ragged rest: inside the
    // loop each stage's wait is then passed on every way round, whatever the trip count.
    int s0 = 0;
    for (; s0 + NBUF <= tA; s0 += NBUF) {
#pragma unroll
        for (int bi = 0; bi < NBUF; ++bi) stage(s0 + bi, bi, std::false_type{});
    }
    static_assert(NBUF == 2, "the ragged rest is taken to be one stage, the last");
    if (s0 < tA) stage(s0, 0, std::true_type{});
    // The index loads are invisible to the compiler, which is free to give their destination registers to something
    // else from here on.  Every set asked for has been waited for by the stage that used it; this wait states it for
    // the whole loop, whatever the trip count, so that nothing of it is in flight when the registers change hands.
    if constexpr (IDX) wait_vmcnt<0>();

    // ---- merge the two halves of the landmark range: half 1 hands its state to half 0 through LDS
    // (the merge area lies over the stage buffers: every wave is through with them first).  The lane's coordinates
    // are derived afresh here, so that none of them holds a register across the loop above.
    __syncthreads();
    const int ln = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
    const int hbe = ln >> 5;
    float(*xch)[NO + 2][64] = reinterpret_cast<float(*)[NO + 2][64]>(smem);
    if (half == 1) {
        xch[wt][NO][ln] = mref;
        xch[wt][NO + 1][ln] = lrun;
#pragma unroll
        for (int i = 0; i < 2 * NP; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) xch[wt][i * 16 + r][ln] = oacc[i][r];
    }
    __syncthreads();
    if (half == 0 && tile_live) {
        const float m1 = xch[wt][NO][ln], l1 = xch[wt][NO + 1][ln];
        const float mm = fmaxf(mref, m1);                 // finite: half 0 always holds landmark 0
        const float f0 = __builtin_amdgcn_exp2f(mref - mm), f1 = __builtin_amdgcn_exp2f(m1 - mm);
        float l = lrun * f0 + l1 * f1;
        l += __shfl_xor(l, 32);
        const float inv = 1.0f / l;
        const float g0 = f0 * inv, g1 = f1 * inv;
#pragma unroll
        for (int i = 0; i < 2 * NP; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[i][r] = oacc[i][r] * g0 + xch[wt][i * 16 + r][ln] * g1;
        const int me = tile * 32 + (ln & 31);             // this lane's query row of the head
        if (me < M) {
            // one workgroup per landmark range: the result; several: a partial row [D values, maximum, denominator, pad]
            int ge = g;                                   // (a fresh division: the first one's reciprocal is not kept)
            asm volatile("" : "+s"(ge));
            const size_t rowid = (size_t)(me / ge) * Hq + (h * ge + me % ge);
            float *orow = splits == 1 ? O + rowid * D : partial + ((size_t)sp * N * Hq + rowid) * (D + 4);
#pragma unroll
            for (int p = 0; p < 2 * NP; ++p)
#pragma unroll
                for (int b = 0; b < 4; ++b)      // registers 4b .. 4b+3 of tile p: dimensions 32 p + 8 b + 4 hb + 0 .. 3
                    *reinterpret_cast<float4 *>(orow + 32 * p + 8 * b + 4 * hbe) =
                        make_float4(oacc[p][4 * b], oacc[p][4 * b + 1], oacc[p][4 * b + 2], oacc[p][4 * b + 3]);
            if (splits > 1 && hbe == 0) *reinterpret_cast<float2 *>(orow + D) = make_float2(mm, l);
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
