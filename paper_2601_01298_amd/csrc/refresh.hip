// Density refresh after the context has grown by m rows (Warp-Cortex Sec. 4: the main stream
// re-extracts landmarks inside its decode loop, so the density must follow a cache that grows by a
// row per step).  L*rho is a plain sum of Gaussian kernel values: the m new keys add one kernel
// column each to the old keys' sums, and their own sums are column sums over all L keys.  That is
// one pass over K -- O(L m d), HBM-bound for small m -- instead of the O(L^2 d) sweep.
//   append_sweep   a workgroup per 2048-key tile of one head; the m new rows sit in LDS as fp32;
//                  a lane group per key row (16-byte loads, 4 rows in flight), squared distances by
//                  direct differences in fp32, exp2; what the new rows add to each old key waits in LDS
//                  and the tile's refreshed densities are written in one coalesced pass at the end (a
//                  4-byte load and store per row group inside the loop cost 13 %: each iteration then
//                  waits on memory twice); column sums leave as one partial per (tile, new row);
//   append_finish  adds the partials of each new row in tile order (deterministic) and writes the
//                  m new densities.
#include "ws_internal.h"

namespace ws {

namespace {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

constexpr int kAppTile = 2048;
constexpr int kAppMaxM = 32;

constexpr int kAppChunk = 768;               // heads per launch: their scales travel as a kernel argument (3 KB)

struct AppScale {
    float s[kAppChunk];     // 0.5 * log2(e) / sigma^2 per head of the chunk
};

template <bool BF16>
__device__ __forceinline__ void widen16(const uint4 &q, float *f)
{
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
    if constexpr (BF16) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            f[2 * j] = __uint_as_float(w[j] << 16);
            f[2 * j + 1] = __uint_as_float(w[j] & 0xFFFF0000u);
        }
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) f[j] = __uint_as_float(w[j]);
    }
}

template <bool BF16, int D>
__global__ void __launch_bounds__(256)
append_sweep(const void *__restrict__ Kv, const float *__restrict__ rho_old, float *__restrict__ rho_new,
             float *__restrict__ colpart, AppScale sc, int head0, int L, int m, int nblk)
{
    constexpr int ES = BF16 ? 2 : 4;
    constexpr int PER = 16 / ES;
    constexpr int LPR = D / PER;
    constexpr int RP = 256 / LPR;
    constexpr int UN = 4;
    __shared__ float nr[kAppMaxM][D];        // the new rows, widened
    __shared__ float cs[kAppMaxM][RP];       // column sums, one slot per row group
    __shared__ float added[kAppTile];        // what the new rows add to each old key of the tile

    const int h = head0 + blockIdx.y, blk = blockIdx.x;
    const int tid = threadIdx.x, sub = tid % LPR, rsub = tid / LPR;
    const char *Kh = reinterpret_cast<const char *>(Kv) + (size_t)h * L * D * ES;
    const int Lold = L - m;
    const float s2 = sc.s[blockIdx.y];

    for (int q = tid; q < m * LPR; q += 256) {
        const int r = q / LPR, c = q % LPR;
        const uint4 v = *reinterpret_cast<const uint4 *>(Kh + ((size_t)(Lold + r) * D + c * PER) * ES);
        widen16<BF16>(v, &nr[r][c * PER]);
    }
    for (int q = tid; q < kAppMaxM * RP; q += 256) cs[q / RP][q % RP] = 0.0f;
    __syncthreads();

    const int lo = blk * kAppTile, hi = min(L, lo + kAppTile);
    for (int r0 = lo; r0 < hi; r0 += UN * RP) {
        uint4 q[UN];
        float x[UN][PER], add[UN];
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int i = min(r0 + u * RP + rsub, hi - 1);
            // the keys stream through once: loads marked non-temporal keep them from displacing anything cached
            const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(Kh + ((size_t)i * D + sub * PER) * ES));
            q[u] = make_uint4(v.x, v.y, v.z, v.w);
        }
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            widen16<BF16>(q[u], x[u]);
            add[u] = 0.0f;
        }
        for (int r = 0; r < m; ++r) {
            float y[PER];
#pragma unroll
            for (int e = 0; e < PER; ++e) y[e] = nr[r][sub * PER + e];
            float col = 0.0f;
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                float acc = 0.0f;
#pragma unroll
                for (int e = 0; e < PER; ++e) {
                    const float t = x[u][e] - y[e];
                    acc = fmaf(t, t, acc);
                }
                acc = lane_group_sum<LPR>(acc);
                const float w = (r0 + u * RP + rsub < hi) ? __builtin_amdgcn_exp2f(-acc * s2) : 0.0f;
                add[u] += w;
                col += w;
            }
            if (sub == 0) cs[r][rsub] += col;          // slot private to this row group
        }
        if (sub == 0) {
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const int i = r0 + u * RP + rsub;
                if (i < hi) added[i - lo] = add[u];
            }
        }
    }
    __syncthreads();
    // the old keys' refreshed densities, a whole tile at a time: consecutive threads, consecutive keys
    for (int i = lo + tid; i < min(hi, Lold); i += 256)
        rho_new[(size_t)h * L + i] = (rho_old[(size_t)h * Lold + i] * (float)Lold + added[i - lo]) / (float)L;
    if (tid < m) {
        float t = 0.0f;
        for (int g = 0; g < RP; ++g) t += cs[tid][g];
        colpart[((size_t)blockIdx.y * nblk + blk) * kAppMaxM + tid] = t;
    }
}

__global__ void __launch_bounds__(64)
append_finish(const float *__restrict__ colpart, float *__restrict__ rho_new, int head0, int L, int m, int nblk)
{
    const int r = threadIdx.x;
    if (r >= m) return;
    float t = 0.0f;
    for (int b = 0; b < nblk; ++b) t += colpart[((size_t)blockIdx.x * nblk + b) * kAppMaxM + r];
    rho_new[(size_t)(head0 + blockIdx.x) * L + (L - m) + r] = t / (float)L;
}

template <bool BF16, int D>
void run_chunk(const void *K, const float *rho_old, float *rho_new, float *colpart, const AppScale &sc, int head0,
               int nh, int L, int m, int nblk, hipStream_t st)
{
    hipLaunchKernelGGL((append_sweep<BF16, D>), dim3(nblk, nh), dim3(256), 0, st, K, rho_old, rho_new, colpart, sc,
                       head0, L, m, nblk);
    hipLaunchKernelGGL(append_finish, dim3(nh), dim3(64), 0, st, colpart, rho_new, head0, L, m, nblk);
}

}  // namespace

int append_max_rows() { return kAppMaxM; }

size_t append_workspace_bytes(int H, int L)
{
    const int nblk = (L + kAppTile - 1) / kAppTile;
    const int nh = H < kAppChunk ? H : kAppChunk;
    return round_up((size_t)nh * nblk * kAppMaxM * sizeof(float), 256);
}

hipError_t launch_density_append(const void *K, bool bf16, int H, int L, int d, int m, const float *sigma_host,
                                 const float *rho_old, float *rho_new, void *ws, hipStream_t st)
{
    const int nblk = (L + kAppTile - 1) / kAppTile;
    float *colpart = reinterpret_cast<float *>(ws);
    for (int h0 = 0; h0 < H; h0 += kAppChunk) {
        const int nh = (H - h0 < kAppChunk) ? H - h0 : kAppChunk;
        AppScale sc;
        for (int i = 0; i < kAppChunk; ++i) {
            const double sg = (i < nh) ? (double)sigma_host[h0 + i] : 1.0;
            sc.s[i] = (float)(0.5 * 1.4426950408889634 / (sg * sg));
        }
        // the chunks share the partial-sum array: they run in order on the one stream
        if (bf16) {
            if (d == 64) run_chunk<true, 64>(K, rho_old, rho_new, colpart, sc, h0, nh, L, m, nblk, st);
            else run_chunk<true, 128>(K, rho_old, rho_new, colpart, sc, h0, nh, L, m, nblk, st);
        } else {
            if (d == 64) run_chunk<false, 64>(K, rho_old, rho_new, colpart, sc, h0, nh, L, m, nblk, st);
            else run_chunk<false, 128>(K, rho_old, rho_new, colpart, sc, h0, nh, L, m, nblk, st);
        }
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace ws
