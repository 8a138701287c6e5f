// Referential injection, cache side (Warp-Cortex Sec. 3.6): rows computed for a side agent's
// thought are appended to the main agent's K/V cache in place; the keys are first rotated by RoPE
// at virtual positions given by the caller, the values are copied.
//   rope_table   cos/sin of pos[r] * base^(-2c/d) for the m positions, angle and sine/cosine in
//                float64 so that large virtual positions lose nothing, stored as fp32 pairs;
//   inject_rows  one thread per 16-byte piece of the lower half of a row and its partner piece in
//                the upper half: rotate, round once to the cache's element type, store; the matching
//                pieces of V are copied.
#include "ws_internal.h"

namespace ws {

namespace {

__global__ void __launch_bounds__(256)
rope_table(const int32_t *__restrict__ pos, int m, int d, double base, float2 *__restrict__ tab)
{
    const int half = d / 2;
    const int g = blockIdx.x * 256 + threadIdx.x;
    if (g >= m * half) return;
    const int r = g / half, c = g - r * half;
    const double ang = (double)pos[r] * pow(base, -2.0 * (double)c / (double)d);
    double sn, cs;
    sincos(ang, &sn, &cs);
    tab[g] = make_float2((float)cs, (float)sn);
}

template <bool BF16>
__global__ void __launch_bounds__(256)
inject_rows(void *__restrict__ Kc, void *__restrict__ Vc, const void *__restrict__ Knew,
            const void *__restrict__ Vnew, const float2 *__restrict__ tab, int H, int Lcap, int d, int L, int m,
            long long total)
{
    constexpr int ES = BF16 ? 2 : 4;
    constexpr int PER = 16 / ES;
    const int half = d / 2, ppr = half / PER;            // thread pieces per row
    const long long g = (long long)blockIdx.x * 256 + threadIdx.x;
    if (g >= total) return;
    const int p = (int)(g % ppr);
    const long long hr = g / ppr;                        // h*m + r
    const int r = (int)(hr % m);
    const long long h = hr / m;
    const size_t src = ((size_t)hr * d + (size_t)p * PER) * ES;
    const size_t dst = (((size_t)h * Lcap + (size_t)(L + r)) * d + (size_t)p * PER) * ES;
    const uint4 lo = *reinterpret_cast<const uint4 *>(reinterpret_cast<const char *>(Knew) + src);
    const uint4 hi = *reinterpret_cast<const uint4 *>(reinterpret_cast<const char *>(Knew) + src + (size_t)half * ES);
    float x0[PER], x1[PER];
    const uint32_t a[4] = {lo.x, lo.y, lo.z, lo.w}, b[4] = {hi.x, hi.y, hi.z, hi.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if constexpr (BF16) {
            x0[2 * j] = __uint_as_float(a[j] << 16);
            x0[2 * j + 1] = __uint_as_float(a[j] & 0xFFFF0000u);
            x1[2 * j] = __uint_as_float(b[j] << 16);
            x1[2 * j + 1] = __uint_as_float(b[j] & 0xFFFF0000u);
        } else {
            x0[j] = __uint_as_float(a[j]);
            x1[j] = __uint_as_float(b[j]);
        }
    }
    float y0[PER], y1[PER];
#pragma unroll
    for (int e = 0; e < PER; ++e) {
        const float2 cs = tab[(size_t)r * half + p * PER + e];
        y0[e] = x0[e] * cs.x - x1[e] * cs.y;
        y1[e] = x1[e] * cs.x + x0[e] * cs.y;
    }
    uint4 olo, ohi;
    if constexpr (BF16) {
        uint32_t wl[4], wh[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            wl[j] = bf16_rne(y0[2 * j]) | (bf16_rne(y0[2 * j + 1]) << 16);
            wh[j] = bf16_rne(y1[2 * j]) | (bf16_rne(y1[2 * j + 1]) << 16);
        }
        olo = make_uint4(wl[0], wl[1], wl[2], wl[3]);
        ohi = make_uint4(wh[0], wh[1], wh[2], wh[3]);
    } else {
        olo = make_uint4(__float_as_uint(y0[0]), __float_as_uint(y0[1]), __float_as_uint(y0[2]), __float_as_uint(y0[3]));
        ohi = make_uint4(__float_as_uint(y1[0]), __float_as_uint(y1[1]), __float_as_uint(y1[2]), __float_as_uint(y1[3]));
    }
    *reinterpret_cast<uint4 *>(reinterpret_cast<char *>(Kc) + dst) = olo;
    *reinterpret_cast<uint4 *>(reinterpret_cast<char *>(Kc) + dst + (size_t)half * ES) = ohi;
    *reinterpret_cast<uint4 *>(reinterpret_cast<char *>(Vc) + dst) =
        *reinterpret_cast<const uint4 *>(reinterpret_cast<const char *>(Vnew) + src);
    *reinterpret_cast<uint4 *>(reinterpret_cast<char *>(Vc) + dst + (size_t)half * ES) =
        *reinterpret_cast<const uint4 *>(reinterpret_cast<const char *>(Vnew) + src + (size_t)half * ES);
}

}  // namespace

size_t inject_workspace_bytes(int d, int m) { return round_up((size_t)m * (d / 2) * sizeof(float2), 256); }

hipError_t launch_inject(void *Kc, void *Vc, bool bf16, int H, int Lcap, int d, int L, const void *Knew,
                         const void *Vnew, int m, const int32_t *pos, float base, void *ws, hipStream_t st)
{
    float2 *tab = reinterpret_cast<float2 *>(ws);
    const int half = d / 2;
    hipLaunchKernelGGL(rope_table, dim3((m * half + 255) / 256), dim3(256), 0, st, pos, m, d, (double)base, tab);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int per = bf16 ? 8 : 4;
    const long long total = (long long)H * m * (half / per);
    const long long blocks = (total + 255) / 256;
    if (blocks > 0x7FFFFFFFLL) return hipErrorInvalidValue;
    if (bf16)
        hipLaunchKernelGGL(inject_rows<true>, dim3((unsigned)blocks), dim3(256), 0, st, Kc, Vc, Knew, Vnew, tab, H, Lcap,
                           d, L, m, total);
    else
        hipLaunchKernelGGL(inject_rows<false>, dim3((unsigned)blocks), dim3(256), 0, st, Kc, Vc, Knew, Vnew, tab, H, Lcap,
                           d, L, m, total);
    return hipGetLastError();
}

}  // namespace ws
