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
#include "ws_internal.h"

namespace ws {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;

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

// One workgroup = 4 waves = 2 query tiles of one KV head x 2 halves of the landmark range; the
// workgroups of a head are placed on the same accelerator die so its K_S/V_S rows are read from HBM
// once and from that die's L2 otherwise.  The two halves run the online softmax independently and
// are merged through LDS at the end: that gives every SIMD the same number of equally long waves
// (at 100 agents a head has 4 query tiles; without the split some SIMDs would carry two of them
// and some one).  The kernel is bound by vector-ALU issue (softmax and operand shuffling), not by
// the MFMAs or by memory, so the per-tile instruction count is what is optimised:
//   - the score scale is folded into the exponent's FMA, the tile maximum is taken on raw scores;
//   - the running maximum is only moved when a tile exceeds it by more than 2^8, so the
//     accumulator is rescaled a few times per query instead of once per tile (weights stay below
//     2^8, harmless in fp32 and in the bf16 hi+lo split);
//   - packed conversions (v_cvt_pk_bf16_f32) and byte permutes (v_perm_b32) build the MFMA operands;
//   - K and V operands of the next landmark tile are requested one tile ahead.
template <int D>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, D == 64 ? 3 : 2)))
attend_bf16(const uint16_t *__restrict__ Q, const uint16_t *__restrict__ Ks, const uint16_t *__restrict__ Vs,
            float *__restrict__ O, int N, int Hq, int Hkv, int k, float scale_log2, int parts)
{
    constexpr int NK = D / 16;   // k-steps of the score product
    constexpr int NP = D / 64;   // 64-wide spans of head dimensions, each an even and an odd tile
    // workgroup id -> (head, part): parts of one head sit on one die (ids are dealt to the 8 dies round-robin)
    int h, part;
    if ((Hkv & 7) == 0) {
        const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
        h = (j / parts) * 8 + xcd;
        part = j % parts;
    } else {
        h = blockIdx.x / parts;
        part = blockIdx.x % parts;
    }
    const int g = Hq / Hkv;
    const int M = N * g;         // query rows that read this KV head
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, nq = lane & 31, hb = lane >> 5;
    const uint16_t *Kh = Ks + (size_t)h * k * D;
    const uint16_t *Vh = Vs + (size_t)h * k * D;
    constexpr int NO = 2 * NP * 16;
    __shared__ float xch[2][NO + 2][64];
    const int wt = wave & 1, half = wave >> 1;
    const int tile = part * 2 + wt;
    const bool tile_live = tile * 32 < M;    // wave-uniform
    const int m = tile * 32 + nq;
    const bool valid = m < M;
    const int mc = valid ? m : M - 1;
    const int agent = mc / g, qh = h * g + mc % g;

    const uint16_t *qrow = Q + ((size_t)agent * Hq + qh) * D;
    bf16x8_t qf[NK];
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) qf[kk] = *reinterpret_cast<const bf16x8_t *>(qrow + kk * 16 + hb * 8);

    f32x16_t oacc[2 * NP];
#pragma unroll
    for (int i = 0; i < 2 * NP; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[i][r] = 0.0f;
    float mref = -__builtin_inff();   // reference maximum (log2 units) the weights are taken against
    float lrun = 0.0f;

    const int nT = (k + 31) / 32;
    const int tA = (nT + 1) / 2;
    const int tb = tile_live ? (half ? tA : 0) : 0;
    const int te = tile_live ? (half ? nT : tA) : 0;
    // Operands of the NEXT landmark tile, requested one tile ahead.  K: one 16-byte piece per k-step.
    // V: the 32-bit word holding head dimensions (2 nq, 2 nq + 1) of 16 landmark rows; contraction slot
    // (kk2, hb, e) <-> landmark t0 + mfma_row(8*kk2+e, hb) = t0 + 16 kk2 + 8 (e/4) + 4 hb + e%4.
    bf16x8_t kn[NK];
    uint32_t vn[2][NP][8];
    auto fetch = [&](int t) {
        const int t0 = t * 32;
        if (t0 + 32 <= k) {      // full tile: one base address per lane, constant offsets
            const uint16_t *krow = Kh + (size_t)(t0 + nq) * D + hb * 8;
#pragma unroll
            for (int kk = 0; kk < NK; ++kk) kn[kk] = *reinterpret_cast<const bf16x8_t *>(krow + kk * 16);
            const uint16_t *vbase = Vh + (size_t)(t0 + 4 * hb) * D + 2 * nq;
#pragma unroll
            for (int kk2 = 0; kk2 < 2; ++kk2)
#pragma unroll
                for (int e = 0; e < 8; ++e)
#pragma unroll
                    for (int p = 0; p < NP; ++p)
                        vn[kk2][p][e] = *reinterpret_cast<const uint32_t *>(
                            vbase + (16 * kk2 + 8 * (e >> 2) + (e & 3)) * D + 64 * p);
        } else {                 // ragged last tile: clamp rows into the head (their weights are zero)
            const uint16_t *krow = Kh + (size_t)min(t0 + nq, k - 1) * D + hb * 8;
#pragma unroll
            for (int kk = 0; kk < NK; ++kk) kn[kk] = *reinterpret_cast<const bf16x8_t *>(krow + kk * 16);
#pragma unroll
            for (int kk2 = 0; kk2 < 2; ++kk2)
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const uint16_t *vrow = Vh + (size_t)min(t0 + mfma_row(8 * kk2 + e, hb), k - 1) * D + 2 * nq;
#pragma unroll
                    for (int p = 0; p < NP; ++p) vn[kk2][p][e] = *reinterpret_cast<const uint32_t *>(vrow + 64 * p);
                }
        }
    };
    if (tb < te) fetch(tb);

    for (int t = tb; t < te; ++t) {
        const int t0 = t * 32;
        bf16x8_t kf[NK];
        uint32_t vd[2][NP][8];
#pragma unroll
        for (int kk = 0; kk < NK; ++kk) kf[kk] = kn[kk];
#pragma unroll
        for (int kk2 = 0; kk2 < 2; ++kk2)
#pragma unroll
            for (int p = 0; p < NP; ++p)
#pragma unroll
                for (int e = 0; e < 8; ++e) vd[kk2][p][e] = vn[kk2][p][e];
        if (t + 1 < te) fetch(t + 1);

        // ---- S^T tile: rows = landmarks t0..t0+31, columns = queries
        f32x16_t sacc;
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[r] = 0.0f;
#pragma unroll
        for (int kk = 0; kk < NK; ++kk) sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], qf[kk], sacc, 0, 0, 0);
        if (t0 + 32 > k) {       // ragged last tile: landmarks past k get zero weight
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
        float psum = 0.0f;
        const float nmref = -mref;
#pragma unroll
        for (int w = 0; w < 8; ++w) {
            f32x2_t pv;
            pv[0] = __builtin_amdgcn_exp2f(fmaf(sacc[2 * w], scale_log2, nmref));
            pv[1] = __builtin_amdgcn_exp2f(fmaf(sacc[2 * w + 1], scale_log2, nmref));
            psum += pv[0] + pv[1];
            const uint32_t hi = __builtin_bit_cast(uint32_t, __builtin_convertvector(pv, bf16x2_t));
            f32x2_t rest;
            rest[0] = pv[0] - __uint_as_float(hi << 16);
            rest[1] = pv[1] - __uint_as_float(hi & 0xFFFF0000u);
            pkh[w] = hi;
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
    }

    // ---- merge the two halves of the landmark range: half 1 hands its state to half 0 through LDS
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
            float *orow = O + ((size_t)agent * Hq + qh) * D;
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
        }
    }
}

template <int D>
__global__ void __launch_bounds__(64)
attend_f32(const float *__restrict__ Q, const float *__restrict__ Ks, const float *__restrict__ Vs,
           float *__restrict__ O, int Hq, int Hkv, int k, float scale)
{
    constexpr int NC = D / 64;   // output dims per lane
    __shared__ float ps[64];
    __shared__ float qs[D];
    const int lane = threadIdx.x;
    const int nq = blockIdx.x;             // agent * Hq + query head
    const int q = nq % Hq;
    const int h = q / (Hq / Hkv);
    const float *qrow = Q + (size_t)nq * D;
    const float *Kh = Ks + (size_t)h * k * D;
    const float *Vh = Vs + (size_t)h * k * D;
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
        if (t < k) {
            const float *kr = Kh + (size_t)t * D;
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
        float psum = p;
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) psum += __shfl_xor(psum, o);
        lrun = lrun * corr + psum;
        __syncthreads();
        const int cnt = min(64, k - c0);
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            float acc = oacc[c] * corr;
            for (int j = 0; j < cnt; ++j) acc = fmaf(ps[j], Vh[(size_t)(c0 + j) * D + lane + 64 * c], acc);
            oacc[c] = acc;
        }
    }
#pragma unroll
    for (int c = 0; c < NC; ++c) O[(size_t)nq * D + lane + 64 * c] = oacc[c] / lrun;
}

}  // namespace

hipError_t launch_attend(const void *Q, const void *Ks, const void *Vs, bool bf16, int N, int Hq, int Hkv, int k,
                         int d, float scale, float *O, hipStream_t st)
{
    if (bf16) {
        const int g = Hq / Hkv;
        const long long M = (long long)N * g;
        const long long parts = (M + 63) / 64;                 // workgroups (2 query tiles each) per head
        const long long blocks = parts * Hkv;
        if (blocks > 0x7FFFFFFFLL) return hipErrorInvalidValue;
        const dim3 grid((unsigned)blocks);
        const float sl2 = scale * 1.4426950408889634f;
        const uint16_t *q = reinterpret_cast<const uint16_t *>(Q);
        const uint16_t *ks = reinterpret_cast<const uint16_t *>(Ks);
        const uint16_t *vs = reinterpret_cast<const uint16_t *>(Vs);
        if (d == 64)
            hipLaunchKernelGGL(attend_bf16<64>, grid, dim3(256), 0, st, q, ks, vs, O, N, Hq, Hkv, k, sl2, (int)parts);
        else if (d == 128)
            hipLaunchKernelGGL(attend_bf16<128>, grid, dim3(256), 0, st, q, ks, vs, O, N, Hq, Hkv, k, sl2, (int)parts);
        else
            return hipErrorInvalidValue;
    } else {
        const long long blocks = (long long)N * Hq;
        if (blocks > 0x7FFFFFFFLL) return hipErrorInvalidValue;
        const float *q = reinterpret_cast<const float *>(Q);
        const float *ks = reinterpret_cast<const float *>(Ks);
        const float *vs = reinterpret_cast<const float *>(Vs);
        if (d == 64)
            hipLaunchKernelGGL(attend_f32<64>, dim3((unsigned)blocks), dim3(64), 0, st, q, ks, vs, O, Hq, Hkv, k, scale);
        else if (d == 128)
            hipLaunchKernelGGL(attend_f32<128>, dim3((unsigned)blocks), dim3(64), 0, st, q, ks, vs, O, Hq, Hkv, k, scale);
        else
            return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace ws
