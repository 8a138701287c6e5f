// Gaussian kernel density of the keys of each head (the inverse-kernel-density ingredient of
// the hybrid landmark score; Warp-Cortex Sec. 2 first paragraph and Sec. 3.3):
//     rho_i = (1/L) sum_j exp(-|k_i - k_j|^2 / (2 sigma^2)).
//
// The L x L sweep is a dense contraction and runs on the matrix cores.  With n_i = |k_i|^2,
//     -|k_i - k_j|^2 / 2 = k_i . k_j - n_i/2 - n_j/2,
// and both norm terms are folded INTO the contraction: every key carries a 16-byte side
// record that extends its row by a few extra columns holding -n/2 split into exactly
// representable pieces next to columns of ones, so the MFMA accumulator leaves the matrix
// core already holding -|k_i - k_j|^2/2.  The epilogue per pair is then one multiply by
// log2(e)/sigma^2, one v_exp_f32 and one add into a per-lane row accumulator: the sweep is
// bound by the vector/transcendental pipe, not by the matrix pipe, so every instruction
// removed there counts.  Padded key slots (index >= L) carry -1e30 in their record, which
// drives their kernel value to exactly 0.  The exponent is formed from fp32 accumulators of
// magnitude ~|k|^2, so a kernel term carries a relative error of about eps_fp32 * |k|^2 / sigma^2:
// fine for bandwidths comparable to the spread of the cloud, meaningless for sigma -> 0 (where
// only the exactly-handled self term survives anyway).
//
// Work split: one workgroup (4 waves) owns RT*32 rows whose MFMA A-fragments stay in
// registers for the whole sweep; the 4 waves stride over the 32-column tiles of the head and
// read B-fragments straight from global memory/L2 in MFMA operand layout (each lane a 16-byte
// piece of one key row), one tile ahead of use.  No LDS, no barrier inside the sweep.
#include "ws_internal.h"

namespace ws {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

// ------------------------------------------------------------------------------------------
// Element traits: how a 32 x KSTEP operand fragment is fetched and multiplied.
// Lane l of a wave supplies row (l % 32) of the tile and the k-slice selected by (l / 32).
// Both operands of K K^T are fetched with the same pattern, so the result does not depend on
// how the hardware orders the k-slots inside an instruction.
// ------------------------------------------------------------------------------------------
struct Bf16Tr {
    typedef uint16_t Elem;
    typedef bf16x8_t Frag;
    static constexpr int KSTEP = 16;  // v_mfma_f32_32x32x16_bf16
    static constexpr int NEXT = 1;    // one extra k-step carries both norm terms
    static __device__ __forceinline__ Frag load(const Elem *row, int kk, int hb)
    {
        return *reinterpret_cast<const Frag *>(row + kk * 16 + hb * 8);
    }
    // record = 8 bf16: {m1,m2,m3,m4, 1,1,1,1},  m1+..+m4 = -n/2
    static __device__ __forceinline__ Frag ext_a(uint4 rec, int hb, int)
    {
        if (hb) rec = make_uint4(0, 0, 0, 0);
        return __builtin_bit_cast(Frag, rec);
    }
    static __device__ __forceinline__ Frag ext_b(uint4 rec, int hb, int)
    {
        uint4 r = hb ? make_uint4(0, 0, 0, 0) : make_uint4(rec.z, rec.w, rec.x, rec.y);
        return __builtin_bit_cast(Frag, r);
    }
    static __device__ __forceinline__ f32x16_t mfma(Frag a, Frag b, f32x16_t c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ double widen(Elem e)
    {
        return (double)__uint_as_float((uint32_t)e << 16);
    }
};

struct F32Tr {
    typedef float Elem;
    typedef float Frag;
    static constexpr int KSTEP = 2;  // v_mfma_f32_32x32x2_f32
    static constexpr int NEXT = 2;   // hi and lo part of -n/2, one k-step each
    static __device__ __forceinline__ Frag load(const Elem *row, int kk, int hb) { return row[kk * 2 + hb]; }
    // record = 4 floats: {hi, lo, 0, 0},  hi + lo = -n/2
    static __device__ __forceinline__ Frag ext_a(uint4 rec, int hb, int e)
    {
        return hb ? 1.0f : __uint_as_float(e ? rec.y : rec.x);
    }
    static __device__ __forceinline__ Frag ext_b(uint4 rec, int hb, int e)
    {
        return hb ? __uint_as_float(e ? rec.y : rec.x) : 1.0f;
    }
    static __device__ __forceinline__ f32x16_t mfma(Frag a, Frag b, f32x16_t c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ double widen(Elem e) { return (double)e; }
};

__device__ __forceinline__ uint32_t bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

// ------------------------------------------------------------------------------------------
// Prepass: per key, the squared norm in fp64 and its side record; per head, the exponent scale.
// ------------------------------------------------------------------------------------------
struct ScaleChunk {
    float s[256];
};

template <class TR, int D>
__global__ void __launch_bounds__(256)
density_prep(const typename TR::Elem *__restrict__ K, uint4 *__restrict__ ext, float *__restrict__ scale,
             ScaleChunk sc, int head0, int L, int Lpad)
{
    const int h = head0 + blockIdx.y;
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (blockIdx.x == 0 && threadIdx.x == 0) scale[h] = sc.s[blockIdx.y];
    if (j >= Lpad) return;
    uint4 rec;
    if (j < L) {
        const typename TR::Elem *row = K + ((size_t)h * L + j) * D;
        double n = 0.0;
#pragma unroll 8
        for (int c = 0; c < D; ++c) {
            const double x = TR::widen(row[c]);
            n += x * x;
        }
        double x = -0.5 * n;
        if constexpr (sizeof(typename TR::Elem) == 2) {
            uint32_t p[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                p[q] = bf16_rne((float)x);
                x -= (double)__uint_as_float(p[q] << 16);
            }
            rec = make_uint4(p[0] | (p[1] << 16), p[2] | (p[3] << 16), 0x3F803F80u, 0x3F803F80u);
        } else {
            const float hi = (float)x;
            const float lo = (float)(x - (double)hi);
            rec = make_uint4(__float_as_uint(hi), __float_as_uint(lo), 0u, 0u);
        }
    } else {
        // padded slot: -1e30 makes exp2() of the pair exactly 0
        if constexpr (sizeof(typename TR::Elem) == 2)
            rec = make_uint4(bf16_rne(-1e30f), 0u, 0x3F803F80u, 0x3F803F80u);
        else
            rec = make_uint4(__float_as_uint(-1e30f), 0u, 0u, 0u);
    }
    ext[(size_t)h * Lpad + j] = rec;
}

// ------------------------------------------------------------------------------------------
// Main sweep.
// ------------------------------------------------------------------------------------------
template <class TR, int D, int RT>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
density_sweep(const typename TR::Elem *__restrict__ K, const uint4 *__restrict__ ext,
              const float *__restrict__ scale, float *__restrict__ rho, int L, int Lpad, int nRB, int total)
{
    typedef typename TR::Frag Frag;
    typedef typename TR::Elem Elem;
    constexpr int NK = D / TR::KSTEP;
    constexpr int NS = NK + TR::NEXT;
    constexpr int BM = RT * 32;
    __shared__ float red[4][BM];

    const int logical = xcd_contiguous(blockIdx.x, total);
    const int h = logical / nRB;
    const int rb = logical - h * nRB;
    const Elem *Kh = K + (size_t)h * L * D;
    const uint4 *exth = ext + (size_t)h * Lpad;
    const float s = scale[h];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 31, hb = lane >> 5;

    // A fragments: RT tiles of 32 rows, resident for the whole sweep
    Frag a[RT][NS];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        const int row = rb * BM + rt * 32 + n;          // < Lpad
        const Elem *rp = Kh + (size_t)min(row, L - 1) * D;
#pragma unroll
        for (int kk = 0; kk < NK; ++kk) a[rt][kk] = TR::load(rp, kk, hb);
        const uint4 rec = exth[row];
#pragma unroll
        for (int e = 0; e < TR::NEXT; ++e) a[rt][NK + e] = TR::ext_a(rec, hb, e);
    }

    float racc[RT][16];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int r = 0; r < 16; ++r) racc[rt][r] = 0.0f;

    const int nCT = Lpad / 32;
    Frag bcur[NS], bnxt[NS];
    auto load_b = [&](Frag *b, int ct) {
        const int col = ct * 32 + n;
        const Elem *cp = Kh + (size_t)min(col, L - 1) * D;
#pragma unroll
        for (int kk = 0; kk < NK; ++kk) b[kk] = TR::load(cp, kk, hb);
        const uint4 rec = exth[col];
#pragma unroll
        for (int e = 0; e < TR::NEXT; ++e) b[NK + e] = TR::ext_b(rec, hb, e);
    };

    int ct = wave;
    if (ct < nCT) load_b(bcur, ct);
    for (; ct < nCT; ct += 4) {
        const bool more = ct + 4 < nCT;     // wave-uniform
        if (more) load_b(bnxt, ct + 4);
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            f32x16_t acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
#pragma unroll
            for (int kk = 0; kk < NS; ++kk) acc = TR::mfma(a[rt][kk], bcur[kk], acc);
            if (ct == rb * RT + rt) {
                // diagonal tile: a key's distance to itself is exactly 0, whatever the rounding of
                // the contraction says (the self term dominates rho for isolated keys)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (8 * (r >> 2) + 4 * hb + (r & 3) == n) acc[r] = 0.0f;
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) racc[rt][r] += __builtin_amdgcn_exp2f(acc[r] * s);
        }
        if (more) {
#pragma unroll
            for (int kk = 0; kk < NS; ++kk) bcur[kk] = bnxt[kk];
        }
    }

    // Row sums: lanes of one half-wave hold the 32 columns of the same rows.
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float v = racc[rt][r];
            v += __shfl_xor(v, 1);
            v += __shfl_xor(v, 2);
            v += __shfl_xor(v, 4);
            v += __shfl_xor(v, 8);
            v += __shfl_xor(v, 16);
            if (n == 0) red[wave][rt * 32 + 8 * (r >> 2) + 4 * hb + (r & 3)] = v;
        }
    __syncthreads();
    if (threadIdx.x < BM) {
        const int row = rb * BM + threadIdx.x;
        if (row < L) {
            const float t = ((red[0][threadIdx.x] + red[1][threadIdx.x]) + red[2][threadIdx.x]) + red[3][threadIdx.x];
            rho[(size_t)h * L + row] = t / (float)L;
        }
    }
}

// ------------------------------------------------------------------------------------------
size_t density_workspace_bytes(int H, int L)
{
    return round_up((size_t)H * sizeof(float), 256) + (size_t)H * density_lpad(L) * sizeof(uint4);
}

template <class TR, int D, int RT>
static hipError_t run(const void *K, int H, int L, const float *sigma_host, float *rho, void *ws, hipStream_t st)
{
    typedef typename TR::Elem Elem;
    const int Lpad = density_lpad(L);
    float *scale = reinterpret_cast<float *>(ws);
    uint4 *ext = reinterpret_cast<uint4 *>(reinterpret_cast<char *>(ws) + round_up((size_t)H * sizeof(float), 256));
    for (int h0 = 0; h0 < H; h0 += 256) {
        const int nh = (H - h0 < 256) ? H - h0 : 256;
        ScaleChunk sc;
        for (int i = 0; i < 256; ++i) {
            // exponent scale log2(e)/sigma^2, so the sweep can use the hardware exp2
            const double sg = (i < nh) ? (double)sigma_host[h0 + i] : 1.0;
            sc.s[i] = (float)(1.4426950408889634 / (sg * sg));
        }
        dim3 grid((Lpad + 255) / 256, nh);
        hipLaunchKernelGGL((density_prep<TR, D>), grid, dim3(256), 0, st, reinterpret_cast<const Elem *>(K), ext,
                           scale, sc, h0, L, Lpad);
    }
    const int BM = RT * 32;
    const int nRB = (L + BM - 1) / BM;
    const long long total = (long long)nRB * H;
    if (total > 0x7FFFFFFFLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL((density_sweep<TR, D, RT>), dim3((unsigned)total), dim3(256), 0, st,
                       reinterpret_cast<const Elem *>(K), ext, scale, rho, L, Lpad, nRB, (int)total);
    return hipGetLastError();
}

hipError_t launch_density(const void *K, bool bf16, int H, int L, int d, const float *sigma_host, float *rho,
                          void *ws, hipStream_t st)
{
    if (bf16) {
        if (d == 64) return run<Bf16Tr, 64, 4>(K, H, L, sigma_host, rho, ws, st);
        if (d == 128) return run<Bf16Tr, 128, 2>(K, H, L, sigma_host, rho, ws, st);
    } else {
        if (d == 64) return run<F32Tr, 64, 2>(K, H, L, sigma_host, rho, ws, st);
        if (d == 128) return run<F32Tr, 128, 1>(K, H, L, sigma_host, rho, ws, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace ws
