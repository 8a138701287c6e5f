// Validation gate (Warp-Cortex Sec. 3.5): cosine similarity of every side thought's hidden state
// with the main agent's, and the accept decision score >= theta.
// One wave per thought: its row (dm elements) is read once with 16-byte loads when the row pitch
// allows it, the three sums (dot, both squared norms) stay in fp32 and are folded over the wave.
// The main agent's vector is re-read by every wave; it is a few KB and lives in L2.
#include "ws_internal.h"

namespace ws {

namespace {

template <bool BF16>
__device__ __forceinline__ float elem(const void *p, size_t i)
{
    if (BF16) return __uint_as_float((uint32_t)reinterpret_cast<const uint16_t *>(p)[i] << 16);
    return reinterpret_cast<const float *>(p)[i];
}

template <bool BF16>
__device__ __forceinline__ void fold16(const uint4 &a, const uint4 &b, float &dot, float &na, float &nb)
{
    const uint32_t x[4] = {a.x, a.y, a.z, a.w}, y[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if (BF16) {
            const float x0 = __uint_as_float(x[j] << 16), x1 = __uint_as_float(x[j] & 0xFFFF0000u);
            const float y0 = __uint_as_float(y[j] << 16), y1 = __uint_as_float(y[j] & 0xFFFF0000u);
            dot = fmaf(x0, y0, dot);
            dot = fmaf(x1, y1, dot);
            na = fmaf(x0, x0, na);
            na = fmaf(x1, x1, na);
            nb = fmaf(y0, y0, nb);
            nb = fmaf(y1, y1, nb);
        } else {
            const float x0 = __uint_as_float(x[j]), y0 = __uint_as_float(y[j]);
            dot = fmaf(x0, y0, dot);
            na = fmaf(x0, x0, na);
            nb = fmaf(y0, y0, nb);
        }
    }
}

template <bool BF16>
__global__ void __launch_bounds__(256)
gate_rows(const void *__restrict__ hmain, const void *__restrict__ T, int N, int dm, float theta,
          float *__restrict__ score, int32_t *__restrict__ accept, int wide)
{
    constexpr int ES = BF16 ? 2 : 4;
    const int lane = threadIdx.x & 63;
    const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (n >= N) return;                                   // whole waves leave together
    const char *row = reinterpret_cast<const char *>(T) + (size_t)n * dm * ES;
    float dot = 0.0f, nt = 0.0f, nh = 0.0f;
    if (wide) {
        const int pieces = dm * ES / 16;
        const uint4 *r4 = reinterpret_cast<const uint4 *>(row);
        const uint4 *h4 = reinterpret_cast<const uint4 *>(hmain);
        for (int c = lane; c < pieces; c += 64) fold16<BF16>(r4[c], h4[c], dot, nt, nh);
    } else {
        for (int c = lane; c < dm; c += 64) {
            const float x = elem<BF16>(row, c), y = elem<BF16>(hmain, c);
            dot = fmaf(x, y, dot);
            nt = fmaf(x, x, nt);
            nh = fmaf(y, y, nh);
        }
    }
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        dot += __shfl_xor(dot, o);
        nt += __shfl_xor(nt, o);
        nh += __shfl_xor(nh, o);
    }
    if (lane == 0) {
        const float den = __fsqrt_rn(nh) * __fsqrt_rn(nt);
        const float sc = den > 0.0f ? dot / den : 0.0f;
        score[n] = sc;
        accept[n] = sc >= theta ? 1 : 0;
    }
}

}  // namespace

hipError_t launch_gate(const void *hmain, const void *T, bool bf16, int N, int dm, float theta, float *score,
                       int32_t *accept, hipStream_t st)
{
    const int es = bf16 ? 2 : 4;
    const bool wide = ((size_t)dm * es) % 16 == 0 && (reinterpret_cast<uintptr_t>(hmain) & 15) == 0 &&
                      (reinterpret_cast<uintptr_t>(T) & 15) == 0;
    const dim3 grid((unsigned)(((long long)N + 3) / 4)), block(256);
    if (bf16)
        hipLaunchKernelGGL(gate_rows<true>, grid, block, 0, st, hmain, T, N, dm, theta, score, accept, wide ? 1 : 0);
    else
        hipLaunchKernelGGL(gate_rows<false>, grid, block, 0, st, hmain, T, N, dm, theta, score, accept, wide ? 1 : 0);
    return hipGetLastError();
}

}  // namespace ws
