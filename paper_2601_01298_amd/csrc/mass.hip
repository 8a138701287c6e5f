// Attention-mass density proxy (Warp-Cortex Sec. 3.3, "Attention Score Summation").
//
// Per layer, A_i = sum over the layer's query heads of softmax_i(scale * q . K_i): one dot
// product per (query head, cached token), so the keys are read ONCE -- an HBM-bound sweep, against
// the O(L^2 d) of the kernel density it can stand in for.  Two kernels:
//   mass_logits   one workgroup per (2048-token tile, KV head): 16-byte loads of the key rows, a
//                 lane group per row, the dot products of all query heads that share the KV head
//                 from one read; writes the logits (log2 units; staged in LDS, one coalesced pass per
//                 tile) and a (max, sum of exp2) pair per (query head, tile);
//   mass_combine  folds the pairs of a layer's heads into (max, 1/sum) per head, then per token adds
//                 the normalised exponentials over the heads and writes the result to every KV head
//                 of the layer (as A, or as 1/A when it is to serve as the density).
#include "ws_internal.h"

namespace ws {

namespace {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

constexpr int kMassTile = 2048;    // tokens per workgroup of mass_logits
constexpr int kMassMaxHq = 128;    // query heads per layer
constexpr float kLog2e = 1.4426950408889634f;

template <bool BF16>
struct Piece;   // 16 bytes of a row, widened to floats
template <>
struct Piece<true> {
    static constexpr int PER = 8;
    static __device__ __forceinline__ void widen(const uint4 &q, float (&f)[8])
    {
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            f[2 * j] = __uint_as_float(w[j] << 16);
            f[2 * j + 1] = __uint_as_float(w[j] & 0xFFFF0000u);
        }
    }
};
template <>
struct Piece<false> {
    static constexpr int PER = 4;
    static __device__ __forceinline__ void widen(const uint4 &q, float (&f)[4])
    {
        f[0] = __uint_as_float(q.x);
        f[1] = __uint_as_float(q.y);
        f[2] = __uint_as_float(q.z);
        f[3] = __uint_as_float(q.w);
    }
};

// (max, sum of exp2(z - max)) pairs merge associatively; an empty pair is (-inf, 0)
__device__ __forceinline__ void merge(float &m, float &s, float m2, float s2)
{
    const float mn = fmaxf(m, m2);
    const float a = (m > -__builtin_inff()) ? s * __builtin_amdgcn_exp2f(m - mn) : 0.0f;
    const float b = (m2 > -__builtin_inff()) ? s2 * __builtin_amdgcn_exp2f(m2 - mn) : 0.0f;
    m = mn;
    s = a + b;
}

template <bool BF16, int D, int MAXG>
__global__ void __launch_bounds__(256)
mass_logits(const void *__restrict__ Kv, const void *__restrict__ Qv, float *__restrict__ z,
            float2 *__restrict__ part, int L, int g, float scale2 /* scale * log2(e) */, int nblk)
{
    typedef Piece<BF16> P;
    constexpr int PER = P::PER;
    constexpr int ES = BF16 ? 2 : 4;
    constexpr int LPR = D / PER;          // lanes per key row
    constexpr int RP = 256 / LPR;         // rows per pass of the workgroup
    constexpr int UN = 4;                 // rows in flight per lane group
    __shared__ float wm[4][MAXG], wsum[4][MAXG];
    // The logits of the tile wait in LDS and leave in one coalesced pass at the end: a 4-byte store per row group
    // inside the streaming loop costs a memory transaction per 32 bytes.  (Eight query heads per KV head would need
    // 64 KB: those keep the direct stores.)
    constexpr bool STAGE = MAXG <= 4;
    __shared__ float zt[STAGE ? MAXG : 1][STAGE ? kMassTile : 1];

    const int kvh = blockIdx.y, blk = blockIdx.x;
    const int tid = threadIdx.x, sub = tid % LPR, rsub = tid / LPR;
    const char *Kh = reinterpret_cast<const char *>(Kv) + (size_t)kvh * L * D * ES;

    float qf[MAXG][PER];
#pragma unroll
    for (int j = 0; j < MAXG; ++j) {
        const int qh = kvh * g + (j < g ? j : 0);
        const uint4 qq = *reinterpret_cast<const uint4 *>(reinterpret_cast<const char *>(Qv) + ((size_t)qh * D + sub * PER) * ES);
        P::widen(qq, qf[j]);
    }
    float m[MAXG], s[MAXG];
#pragma unroll
    for (int j = 0; j < MAXG; ++j) {
        m[j] = -__builtin_inff();
        s[j] = 0.0f;
    }

    const int lo = blk * kMassTile, hi = min(L, lo + kMassTile);
    for (int r0 = lo; r0 < hi; r0 += UN * RP) {
        uint4 q[UN];
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int i = min(r0 + u * RP + rsub, hi - 1);
            // the keys stream through once: loads marked non-temporal keep them from displacing anything cached
            const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(Kh + ((size_t)i * D + sub * PER) * ES));
            q[u] = make_uint4(v.x, v.y, v.z, v.w);
        }
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int i = r0 + u * RP + rsub;
            float f[PER];
            P::widen(q[u], f);
#pragma unroll
            for (int j = 0; j < MAXG; ++j) {
                if (j < g) {
                    float acc = 0.0f;
#pragma unroll
                    for (int e = 0; e < PER; ++e) acc = fmaf(f[e], qf[j][e], acc);
                    acc = lane_group_sum<LPR>(acc);
                    const float zz = acc * scale2;
                    if (i < hi) {
                        if (sub == 0) {
                            if constexpr (STAGE) zt[j][i - lo] = zz;
                            else z[(size_t)(kvh * g + j) * L + i] = zz;
                        }
                        const float mn = fmaxf(m[j], zz);
                        s[j] = s[j] * __builtin_amdgcn_exp2f(m[j] - mn) + __builtin_amdgcn_exp2f(zz - mn);
                        m[j] = mn;
                    }
                }
            }
        }
    }
    // one lane per row group speaks for its rows; fold the lanes of a wave, then the 4 waves
    const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
    for (int j = 0; j < MAXG; ++j) {
        if (j < g) {
            float mm = (sub == 0) ? m[j] : -__builtin_inff();
            float ss = (sub == 0) ? s[j] : 0.0f;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const float m2 = __shfl_xor(mm, o), s2 = __shfl_xor(ss, o);
                merge(mm, ss, m2, s2);
            }
            if (lane == 0) {
                wm[wave][j] = mm;
                wsum[wave][j] = ss;
            }
        }
    }
    __syncthreads();
    if constexpr (STAGE) {
#pragma unroll
        for (int j = 0; j < MAXG; ++j)
            if (j < g)
                for (int i = lo + tid; i < hi; i += 256) z[(size_t)(kvh * g + j) * L + i] = zt[j][i - lo];
    }
    if (tid < g) {
        float mm = wm[0][tid], ss = wsum[0][tid];
        for (int w = 1; w < 4; ++w) merge(mm, ss, wm[w][tid], wsum[w][tid]);
        part[(size_t)(kvh * g + tid) * nblk + blk] = make_float2(mm, ss);
    }
}

__global__ void __launch_bounds__(256)
mass_combine(const float *__restrict__ z, const float2 *__restrict__ part, float *__restrict__ out, int L, int Hkv,
             int Hq, int nblk, int as_density)
{
    __shared__ float mq[kMassMaxHq], rinv[kMassMaxHq];
    const int grp = blockIdx.y, tid = threadIdx.x;
    for (int q = tid; q < Hq; q += 256) {
        const float2 *p = part + (size_t)(grp * Hq + q) * nblk;
        float mm = -__builtin_inff(), ss = 0.0f;
        for (int b = 0; b < nblk; ++b) merge(mm, ss, p[b].x, p[b].y);
        mq[q] = mm;
        rinv[q] = 1.0f / ss;
    }
    __syncthreads();
    const int i = blockIdx.x * 256 + tid;
    if (i >= L) return;
    float A = 0.0f;
    for (int q = 0; q < Hq; ++q) A += __builtin_amdgcn_exp2f(z[(size_t)(grp * Hq + q) * L + i] - mq[q]) * rinv[q];
    const float v = as_density ? 1.0f / fmaxf(A, 1e-30f) : A;
    for (int hk = 0; hk < Hkv; ++hk) out[(size_t)(grp * Hkv + hk) * L + i] = v;
}

struct MassWs {
    size_t z, part, total;
    int nblk;
};

MassWs mass_layout(int G, int Hq, int L)
{
    MassWs w;
    w.nblk = (L + kMassTile - 1) / kMassTile;
    w.z = 0;
    w.part = round_up((size_t)G * Hq * L * sizeof(float), 256);
    w.total = w.part + round_up((size_t)G * Hq * w.nblk * sizeof(float2), 256);
    return w;
}

template <bool BF16, int D>
void run_logits(const void *K, const void *Q, float *z, float2 *part, int GHkv, int L, int g, float scale2, int nblk,
                hipStream_t st)
{
    const dim3 grid(nblk, GHkv), block(256);
    if (g == 1)
        hipLaunchKernelGGL((mass_logits<BF16, D, 1>), grid, block, 0, st, K, Q, z, part, L, g, scale2, nblk);
    else if (g == 2)
        hipLaunchKernelGGL((mass_logits<BF16, D, 2>), grid, block, 0, st, K, Q, z, part, L, g, scale2, nblk);
    else if (g <= 4)
        hipLaunchKernelGGL((mass_logits<BF16, D, 4>), grid, block, 0, st, K, Q, z, part, L, g, scale2, nblk);
    else
        hipLaunchKernelGGL((mass_logits<BF16, D, 8>), grid, block, 0, st, K, Q, z, part, L, g, scale2, nblk);
}

}  // namespace

bool mass_supported(int Hkv, int Hq) { return Hq % Hkv == 0 && Hq <= kMassMaxHq && Hq / Hkv <= 8; }

size_t mass_workspace_bytes(int G, int Hq, int L) { return mass_layout(G, Hq, L).total; }

hipError_t launch_attention_mass(const void *K, const void *Q, bool bf16, int G, int Hkv, int Hq, int L, int d,
                                 float scale, int as_density, float *out, void *ws, hipStream_t st)
{
    const MassWs w = mass_layout(G, Hq, L);
    char *base = reinterpret_cast<char *>(ws);
    float *z = reinterpret_cast<float *>(base + w.z);
    float2 *part = reinterpret_cast<float2 *>(base + w.part);
    const int g = Hq / Hkv;
    const float scale2 = scale * kLog2e;
    if (bf16) {
        if (d == 64) run_logits<true, 64>(K, Q, z, part, G * Hkv, L, g, scale2, w.nblk, st);
        else run_logits<true, 128>(K, Q, z, part, G * Hkv, L, g, scale2, w.nblk, st);
    } else {
        if (d == 64) run_logits<false, 64>(K, Q, z, part, G * Hkv, L, g, scale2, w.nblk, st);
        else run_logits<false, 128>(K, Q, z, part, G * Hkv, L, g, scale2, w.nblk, st);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(mass_combine, dim3((L + 255) / 256, G), dim3(256), 0, st, z, part, out, L, Hkv, Hq, w.nblk,
                       as_density);
    return hipGetLastError();
}

}  // namespace ws
