// Fill the synapse buffer: copy the chosen K and V rows of every head, in pick order
// (Warp-Cortex Sec. 3.3: the synapse is a shared buffer that holds only the landmarks).
// Pure data movement: each thread moves one 16-byte piece of one row of K and of V, so a row
// (128 or 256 bytes for bf16, 256 or 512 for fp32) is read and written by neighbouring lanes.
#include "ws_internal.h"

namespace ws {

__global__ void __launch_bounds__(256)
gather_rows(const uint4 *__restrict__ K, const uint4 *__restrict__ V, const int32_t *__restrict__ idx,
            uint4 *__restrict__ Ks, uint4 *__restrict__ Vs, int L, int k, int cpr /*16-byte chunks per row*/,
            long long nchunks /* H*k*cpr */)
{
    const long long g = (long long)blockIdx.x * 256 + threadIdx.x;
    if (g >= nchunks) return;
    const long long row = g / cpr;          // h*k + t
    const int c = (int)(g - row * cpr);
    const long long h = row / k;
    int src = idx[row];
    src = src < 0 ? 0 : (src >= L ? L - 1 : src);
    const size_t from = ((size_t)h * L + (size_t)src) * cpr + c;
    Ks[g] = K[from];
    Vs[g] = V[from];
}

hipError_t launch_gather(const void *K, const void *V, int row_bytes, int H, int L, const int32_t *idx, int k,
                         void *Ks, void *Vs, hipStream_t st)
{
    const int cpr = row_bytes / 16;
    const long long nchunks = (long long)H * k * cpr;
    const long long blocks = (nchunks + 255) / 256;
    if (blocks > 0x7FFFFFFFLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(gather_rows, dim3((unsigned)blocks), dim3(256), 0, st, reinterpret_cast<const uint4 *>(K),
                       reinterpret_cast<const uint4 *>(V), idx, reinterpret_cast<uint4 *>(Ks),
                       reinterpret_cast<uint4 *>(Vs), L, k, cpr, nchunks);
    return hipGetLastError();
}

}  // namespace ws
