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
// drives their kernel value to exactly 0.
//
// Accuracy and translation.  The exponent is formed from fp32 accumulators of magnitude ~|k|^2, so
// a kernel term carries a relative error of about 2^-23 |k|^2 / sigma^2.  The density itself does
// not depend on where the cloud sits, but that error does: a cloud with a common offset (what a
// real key cache looks like) would lose accuracy in proportion to the offset squared.  So the
// prepass moves the cloud: per head and coordinate it takes the mid-range c of the keys (rounded to
// bf16) and, WHERE k - c IS EXACTLY A bf16 NUMBER FOR EVERY KEY of that coordinate (decided from the
// coordinate's minimum, maximum and smallest non-zero magnitude: the keys of a coordinate with an
// offset well above its spread all share a coarse grid, so their differences to c need few bits),
// the sweep runs on a copy of the head holding k - c.  That copy is the same cloud, translated: no
// rounding takes part.  Coordinates where the differences are not exact (a spread comparable to the
// offset: little to gain there) keep c = 0; heads with c = 0 throughout are swept in place.  What is
// left is reported: per head the estimate 2^-23 mean|k - c|^2 / sigma^2 is written to the head of the
// workspace, and a flag is raised when it exceeds kErrBound (bandwidths far below the cloud's spread,
// offsets that cannot be removed exactly).  For sigma -> 0 only the self term survives, and that one
// is exact by construction.
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

// ------------------------------------------------------------------------------------------
// Prepass.
//   density_stats   (bf16)  per head, coordinate and chunk of rows: minimum, maximum, smallest non-zero magnitude
//   density_decide          per head: the reference point c (zero where k - c would not be exact), which copy of the
//                           head the sweep reads, the exponent scale; clears the flag
//   density_prep            per key: k - c written to the copy (heads that move), |k - c|^2 in fp64 and its side
//                           record; per block of 256 keys the sum of the squared norms
//   density_estimate        per head: 2^-23 mean|k - c|^2 / sigma^2, and the flag
// ------------------------------------------------------------------------------------------
struct ScaleChunk {
    float s[256];
};

constexpr int kStatChunks = 16;          // row chunks per head in density_stats
constexpr float kErrBound = 2.0e-5f;     // estimated relative error of a kernel term above which a head is flagged

struct PrepWs {
    int *flag;              // [0] = 1 if some head's estimate exceeds kErrBound
    float *est;             // [H] estimated relative error of one kernel term
    float *scale;           // [H] log2(e) / sigma^2
    const void **kbase;     // [H] the rows the sweep reads: the caller's, or the translated copy
    int *cand;              // [H] some coordinate of the head may be moved (after the sample pass); moved (after the full one)
    float *cvec;            // [H][D] reference point
    float *stat;            // [H][kStatChunks][3][D] min, max, smallest non-zero magnitude (bf16 keys only)
    double *nsum;           // [H][Lpad/256] sum of squared norms per block of keys
    uint4 *ext;             // [H][Lpad] side records
    void *Kc;               // [H][L][D] translated copy (bf16 keys only)
    unsigned long long *acc;   // [H][Lpad] kernel sums in fixed point (symmetric sweep only, else NULL): cleared here
};

// Two passes.  Pass 0 looks at the first eighth of every chunk of rows.  More keys only widen a coordinate's range
// and refine its grid, so a coordinate that fails the exactness test on the sample is taken to fail it on the whole
// head (a rule on the safe side: it decides only whether a head is moved, never a value): heads without a candidate
// coordinate are settled by the sample, and pass 1, which reads the rest and merges, skips them.
template <int D>
__global__ void __launch_bounds__(256)
density_stats(const uint16_t *__restrict__ K, float *__restrict__ stat, int L, int pass, const int *__restrict__ cand)
{
    constexpr int CH = D / 8;            // 16-byte pieces per row
    constexpr int RPS = 256 / CH;        // rows per sweep of the block
    __shared__ float red[3][RPS][D + 1];
    const int h = blockIdx.y, chunk = blockIdx.x;
    if (pass == 1 && !cand[h]) return;
    const int per = (L + kStatChunks - 1) / kStatChunks;
    const int cut = chunk * per + (per + 7) / 8;
    const int lo = pass == 0 ? chunk * per : min(L, cut);
    const int hi = pass == 0 ? min(L, cut) : min(L, (chunk + 1) * per);
    const int piece = threadIdx.x % CH, r0 = threadIdx.x / CH;
    float mn[8], mx[8], ma[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        mn[i] = __builtin_inff();
        mx[i] = -__builtin_inff();
        ma[i] = __builtin_inff();
    }
    const uint16_t *Kh = K + (size_t)h * L * D;
    for (int r = lo + r0; r < hi; r += RPS) {
        const uint4 q = *reinterpret_cast<const uint4 *>(Kh + (size_t)r * D + piece * 8);
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float v = __uint_as_float((i & 1) ? (w[i >> 1] & 0xFFFF0000u) : (w[i >> 1] << 16));
            mn[i] = fminf(mn[i], v);
            mx[i] = fmaxf(mx[i], v);
            const float av = fabsf(v);
            if (av > 0.0f) ma[i] = fminf(ma[i], av);
        }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        red[0][r0][piece * 8 + i] = mn[i];
        red[1][r0][piece * 8 + i] = mx[i];
        red[2][r0][piece * 8 + i] = ma[i];
    }
    __syncthreads();
    for (int c = threadIdx.x; c < 3 * D; c += 256) {
        const int which = c / D, j = c % D;
        float v = red[which][0][j];
        for (int r = 1; r < RPS; ++r) v = (which == 1) ? fmaxf(v, red[which][r][j]) : fminf(v, red[which][r][j]);
        float *dst = stat + (((size_t)h * kStatChunks + chunk) * 3 + which) * D + j;
        if (pass == 1) v = (which == 1) ? fmaxf(v, *dst) : fminf(v, *dst);
        *dst = v;
    }
}

// 2^(floor(log2 v) - 7): the spacing of bf16 numbers around |v| (v finite, normal, non-zero)
__device__ __forceinline__ float bf16_ulp(float v)
{
    const uint32_t e = (__float_as_uint(v) >> 23) & 0xFFu;
    return e > 7u ? __uint_as_float((e - 7u) << 23) : 0.0f;
}

template <int D>
__global__ void __launch_bounds__(D)
density_decide(PrepWs w, const void *K, size_t head_bytes, ScaleChunk sc, int head0, int centre)
{
    const int h = head0 + blockIdx.x, j = threadIdx.x;
    float c = 0.0f;
    if (centre) {
        float mn = __builtin_inff(), mx = -__builtin_inff(), ma = __builtin_inff();
        for (int ch = 0; ch < kStatChunks; ++ch) {
            const float *st = w.stat + ((size_t)h * kStatChunks + ch) * 3 * D;
            mn = fminf(mn, st[j]);
            mx = fmaxf(mx, st[D + j]);
            ma = fminf(ma, st[2 * D + j]);
        }
        if (mx >= mn && ma < __builtin_inff()) {          // finite, not all zero
            const float mid = __uint_as_float(bf16_rne(0.5f * mn + 0.5f * mx) << 16);
            if (mid != 0.0f && fabsf(mid) < __builtin_inff()) {
                // every key of the coordinate and c are multiples of g (the finer of their bf16 spacings); k - c is a
                // bf16 number when |k - c| <= 256 g.  g must be a normal number well inside the range.
                const float g = fminf(bf16_ulp(ma), bf16_ulp(mid));
                const float X = fmaxf(mx - mid, mid - mn) * 1.000001f;
                if (g >= 7.0e-31f && X <= 256.0f * g) c = mid;
            }
        }
    }
    w.cvec[(size_t)h * D + j] = c;
    const int moved = __syncthreads_or(c != 0.0f);
    if (j == 0) {
        w.kbase[h] = moved ? (const void *)((const char *)w.Kc + (size_t)h * head_bytes)
                           : (const void *)((const char *)K + (size_t)h * head_bytes);
        w.cand[h] = moved;
        w.scale[h] = sc.s[blockIdx.x];
        if (h == 0) w.flag[0] = 0;
    }
}

template <class TR, int D>
__global__ void __launch_bounds__(256)
density_prep(const typename TR::Elem *__restrict__ K, PrepWs w, int L, int Lpad)
{
    typedef typename TR::Elem Elem;
    constexpr bool kBf16 = sizeof(Elem) == 2;
    __shared__ double part[256];
    const int h = blockIdx.y;
    const int j = blockIdx.x * 256 + threadIdx.x;
    const float *cv = w.cvec + (size_t)h * D;
    const bool moved = kBf16 && w.kbase[h] != (const void *)(K + (size_t)h * L * D);
    uint4 rec;
    double n = 0.0;
    if (j < L) {
        // whole row through 16-byte loads (a thread owns a row: 8 or more loads hit the same lines)
        const uint4 *row = reinterpret_cast<const uint4 *>(K + ((size_t)h * L + j) * D);
        uint4 *crow = reinterpret_cast<uint4 *>(reinterpret_cast<Elem *>(w.Kc) + ((size_t)h * L + j) * D);
        constexpr int PER = 16 / sizeof(Elem);
        constexpr int NPC = D / PER;             // 16-byte pieces per row
        constexpr int GRP = NPC < 8 ? NPC : 8;   // pieces in flight at a time (all loads of a group before any store)
#pragma unroll
        for (int c0 = 0; c0 < NPC; c0 += GRP) {
            uint4 qs[GRP];
#pragma unroll
            for (int c = 0; c < GRP; ++c) qs[c] = row[c0 + c];
#pragma unroll
            for (int c = 0; c < GRP; ++c) {
                Elem e[PER];
                __builtin_memcpy(e, &qs[c], 16);
                uint32_t xb[PER];
#pragma unroll
                for (int i = 0; i < PER; ++i) {
                    if constexpr (kBf16) {
                        // exact: c is non-zero only where every k - c of the coordinate is a bf16 number
                        // (heads that stay in place skip the reference point: it is zero throughout)
                        float xf = __uint_as_float((uint32_t)e[i] << 16);
                        if (moved) xf -= cv[(c0 + c) * PER + i];
                        xb[i] = __float_as_uint(xf) >> 16;
                        n += (double)xf * (double)xf;
                    } else {
                        const double x = TR::widen(e[i]);
                        n += x * x;
                    }
                }
                if constexpr (kBf16) {
                    if (moved)
                        crow[c0 + c] = make_uint4(xb[0] | (xb[1] << 16), xb[2] | (xb[3] << 16), xb[4] | (xb[5] << 16),
                                                  xb[6] | (xb[7] << 16));
                }
            }
        }
        double x = -0.5 * n;
        if constexpr (kBf16) {
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
        if constexpr (kBf16)
            rec = make_uint4(bf16_rne(-1e30f), 0u, 0x3F803F80u, 0x3F803F80u);
        else
            rec = make_uint4(__float_as_uint(-1e30f), 0u, 0u, 0u);
    }
    if (j < Lpad) {
        w.ext[(size_t)h * Lpad + j] = rec;
        // the symmetric sweep's cell of a key starts at its self term, exactly 1 (in 32.32 fixed point): kept out of
        // the fp32 row accumulators, where a 1 would swallow the many kernel values below its half ulp that make
        // up the rest of an isolated key's sum
        if (w.acc) w.acc[(size_t)h * Lpad + j] = (j < L) ? (1ull << 32) : 0ull;
    }
    // sum of the block's squared norms, in a fixed order
    part[threadIdx.x] = n;
    __syncthreads();
    for (int o = 128; o >= 1; o >>= 1) {
        if ((int)threadIdx.x < o) part[threadIdx.x] += part[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) w.nsum[(size_t)h * (Lpad / 256) + blockIdx.x] = part[0];
}

__global__ void __launch_bounds__(256)
density_estimate(PrepWs w, int H, int L, int Lpad)
{
    const int h = blockIdx.x * 256 + threadIdx.x;
    if (h >= H) return;
    double t = 0.0;
    for (int b = 0; b < Lpad / 256; ++b) t += w.nsum[(size_t)h * (Lpad / 256) + b];
    // scale = log2(e) / sigma^2
    const float est = (float)(1.1920928955078125e-7 * (t / (double)L) * ((double)w.scale[h] / 1.4426950408889634));
    w.est[h] = est;
    if (!(est <= kErrBound)) atomicExch(w.flag, 1);
}

// ------------------------------------------------------------------------------------------
// Main sweep.
// ------------------------------------------------------------------------------------------
template <class TR, int D, int RT>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
density_sweep(const void *const *__restrict__ kbase, const uint4 *__restrict__ ext,
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
    const Elem *Kh = reinterpret_cast<const Elem *>(kbase[h]);     // the caller's rows or their translated copy
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


// LDS-only barrier: waits for this wave's LDS traffic, not for its global loads
__device__ __forceinline__ void lds_only_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Asynchronous 16-byte-per-lane copy global -> LDS (no registers in between): lane i of the wave reads base +
// byte_offset and lands at lds_base + 16 * i.  Completion is counted by vmcnt like any vector load; the compiler does not see it, so the
// caller waits explicitly before the barrier that publishes the data.
__device__ __forceinline__ void dma16(const void *base /* wave-uniform */, unsigned byte_offset, const void *lds_base)
{
    const unsigned la =
        __builtin_amdgcn_readfirstlane((unsigned)(size_t)(__attribute__((address_space(3))) const void *)lds_base);
    asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(byte_offset), "s"(base), "s"(la) : "memory", "m0");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// ------------------------------------------------------------------------------------------
// Symmetric sweep (bf16 keys, heads of at least a few row blocks).
//
// The kernel matrix is symmetric, and its cost is the exponential, not the contraction: so every
// unordered pair is evaluated ONCE and its value is added to the row sum of i and to the
// column sum of j.  Keys are cut into blocks of BM rows; workgroup I evaluates block I against
// blocks I (row sums only), I+1 .. I+nBoth (row and column sums) and, when the block count is
// even, I + nB/2 (row sums only; its partner evaluates the transposed copy).  Every workgroup
// does the same amount of work.  Row sums stay in registers for the whole sweep.  Column sums
// of one visited block are reduced over the workgroup's 4 waves in LDS and added to the keys'
// accumulator cells (fixed point, integer atomics: see fixed_add), as are the row sums at the
// end; a last small kernel turns the cells into rho.  Integer addition is associative, so the
// result does not depend on scheduling.
//
// The 4 waves of a workgroup own different rows (RTW tiles of 32 each) and share the stream of
// column tiles: 64 key rows per stage reach the LDS by asynchronous global -> LDS copies (no
// registers in between) issued two stages ahead into three rotating buffers, and are read back in
// MFMA operand layout (16-byte pieces, XOR-swizzled by row so the 8 lanes served per LDS cycle hit
// 8 different bank groups; the swizzle is applied on the global side of the copy).  One LDS-only
// barrier per stage publishes the stage and retires the buffer two stages back.
// ------------------------------------------------------------------------------------------
// The kernel sums of a key come from many workgroups (its own row block, and every block that visits it as
// a column block).  They are accumulated in 32.32 fixed point with integer atomics: integer addition is
// associative, so the result does not depend on the order in which the workgroups arrive (a floating-point
// atomic would), and one 8-byte cell per key replaces a slot per visiting workgroup.  A contribution is a sum
// of at most a few hundred kernel values (<= 1 each), the total at most L < 2^24: no overflow, and the 2^-32
// resolution is far below fp32 rounding of sums that are >= 1 (the self term).
__device__ __forceinline__ void fixed_add(unsigned long long *cell, float v)
{
    const unsigned long long q = (unsigned long long)__float2ll_rn(v * 4294967296.0f);
    __hip_atomic_fetch_add(cell, q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int D, int RTW, bool BOTH, bool DIAG>
__device__ __forceinline__ void sym_tile(const bf16x8_t (&a)[RTW][D / 16 + 1], const bf16x8_t (&b)[D / 16 + 1],
                                         float (&racc)[RTW][16], float &csum, float s, int n, int hb,
                                         int diag_rt /* row tile that meets this column tile, or -1 */)
{
    constexpr int NS = D / 16 + 1;
    // The contraction of row tile rt+1 is issued before the exponentials of row tile rt, one MFMA per
    // slice of the vector work, so the matrix core runs under the vector pipe inside one wave.
    f32x16_t acc[2];
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[0][r] = 0.0f;
#pragma unroll
    for (int kk = 0; kk < NS; ++kk) acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0][kk], b[kk], acc[0], 0, 0, 0);
#pragma unroll
    for (int rt = 0; rt < RTW; ++rt) {
        f32x16_t &cur = acc[rt & 1], &nxt = acc[(rt + 1) & 1];
        if (DIAG && rt == diag_rt) {
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (8 * (r >> 2) + 4 * hb + (r & 3) == n) cur[r] = -1e30f;   // the self term is in the cell already
        }
        if (rt + 1 < RTW) {
#pragma unroll
            for (int r = 0; r < 16; ++r) nxt[r] = 0.0f;
#pragma unroll
            for (int kk = 0; kk < NS; ++kk) {
                nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[rt + 1][kk], b[kk], nxt, 0, 0, 0);
#pragma unroll
                for (int r = (kk * 16 + NS - 1) / NS; r < ((kk + 1) * 16 + NS - 1) / NS; ++r) {
                    const float w = __builtin_amdgcn_exp2f(cur[r] * s);
                    racc[rt][r] += w;
                    if (BOTH) csum += w;
                }
                // keeps each MFMA between its shares of the vector work
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float w = __builtin_amdgcn_exp2f(cur[r] * s);
                racc[rt][r] += w;
                if (BOTH) csum += w;
            }
        }
    }
}

template <int D, int RTW>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu((D == 64 && RTW <= 2) ? 3 : 2, (D == 64 && RTW <= 2) ? 3 : 2)))
density_sym(const void *const *__restrict__ kbase, const uint4 *__restrict__ ext, const float *__restrict__ scale,
            unsigned long long *__restrict__ acc, int L, int Lpad, int nB, int nBoth, int head0, int total)
{
    constexpr int NK = D / 16, NS = NK + 1;
    constexpr int BM = 4 * RTW * 32;       // rows (and columns) per block
    constexpr int CH = D / 8;              // 16-byte pieces per key row
    constexpr int SC = 64;                 // key rows per LDS stage
    constexpr int SPB = BM / SC;           // stages per block
    constexpr int NLD = SC * CH / 256;     // 16-byte pieces each thread moves per stage
    constexpr int NBUF = 3, PF = NBUF - 1;  // LDS buffers in rotation; stages the copies run ahead
    __shared__ uint4 sB[NBUF][SC * CH];
    __shared__ uint4 sE[NBUF][SC];
    __shared__ float cs[4][2][BM];          // column sums of a block: per wave and half-wave

    const int logical = xcd_contiguous(blockIdx.x, total);
    const int hl = logical / nB, I = logical - hl * nB;
    const int h = head0 + hl;
    const uint16_t *Kh = reinterpret_cast<const uint16_t *>(kbase[h]);     // the caller's rows or their translated copy
    const uint4 *exth = ext + (size_t)h * Lpad;
    const float s = scale[h];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31, hb = lane >> 5;

    bf16x8_t a[RTW][NS];
#pragma unroll
    for (int rt = 0; rt < RTW; ++rt) {
        const int row = I * BM + (wave * RTW + rt) * 32 + n;      // < Lpad
        const uint16_t *rp = Kh + (size_t)min(row, L - 1) * D;
#pragma unroll
        for (int kk = 0; kk < NK; ++kk) a[rt][kk] = Bf16Tr::load(rp, kk, hb);
        // the record is {m1..m4, 1,1,1,1} with m1+..+m4 = -n/2: the column side uses it as it is, the row side
        // swaps its halves, so the extra k-step adds -n_i/2 - n_j/2.  Only the first 8 k-slots are used: the row
        // side holds zeros in the others, so what the column side holds there does not matter.
        const uint4 rec = exth[row];
        a[rt][NK] = __builtin_bit_cast(bf16x8_t, hb ? make_uint4(0, 0, 0, 0) : make_uint4(rec.z, rec.w, rec.x, rec.y));
    }
    float racc[RTW][16];
#pragma unroll
    for (int rt = 0; rt < RTW; ++rt)
#pragma unroll
        for (int r = 0; r < 16; ++r) racc[rt][r] = 0.0f;

    const int nblk = 1 + nBoth + ((nB > 1 && (nB & 1) == 0) ? 1 : 0);
    const int nst = nblk * SPB;

    // Key rows reach the LDS by asynchronous copies issued two stages ahead, already in the swizzled order the
    // MFMA operand reads expect (slot c of row r holds piece c ^ (r & 7)); three buffers rotate.
    // per-thread constants of the copy: which row of a stage and which (swizzled) 16-byte piece of it; the
    // thread's further pieces of a stage sit 256 / CH rows below with the same swizzle (256 / CH is a multiple of 8)
    // (byte offsets inside a head are 32-bit: the entry point admits L < 2^24 rows of at most 256 bytes)
    const int crow = tid / CH;
    const unsigned cpiece = (unsigned)(((tid % CH) ^ (crow & 7)) * 16);
    auto issue = [&](int sidx) {
        const int J = (I + sidx / SPB) % nB;
        const int col0 = J * BM + (sidx % SPB) * SC;
        const int bi = sidx % NBUF;
#pragma unroll
        for (int i = 0; i < NLD; ++i)
            dma16(Kh, (unsigned)min(col0 + crow + i * (256 / CH), L - 1) * (unsigned)(D * 2) + cpiece,
                  &sB[bi][wave * 64 + 256 * i]);
        if (wave == 0) dma16(exth, (unsigned)(col0 + lane) * 16u, &sE[bi][0]);
    };

    // LDS read positions of this lane: row n of a tile, the swizzled pieces of the NK k-steps
    const int boff0 = n * CH;
    int bpiece[NK];
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) bpiece[kk] = (2 * kk + hb) ^ (n & 7);
    float *csw = &cs[wave][hb][n];

    // The row operands must be in their registers before the first asynchronous copy is issued: the compiler
    // would otherwise wait for them at their first use inside the loop, with a count that also covers the copies.
    wait_vmcnt<0>();

#pragma unroll
    for (int p = 0; p < PF; ++p)
        if (p < nst) issue(p);
    for (int sidx = 0; sidx < nst; ++sidx) {
        const int buf = sidx % NBUF;
        // this wave's copies of the stage have landed (those of the next stage may still be in flight) ...
        if (sidx + 1 < nst) {
            if (wave == 0) wait_vmcnt<NLD + 1>();
            else wait_vmcnt<NLD>();
        } else {
            wait_vmcnt<0>();
        }
        // ... and so have everybody's; all waves are through with the stage before
        lds_only_barrier();
        if (sidx + PF < nst) issue(sidx + PF);
        const int j = sidx / SPB, sin = sidx - j * SPB;
        const bool both = j >= 1 && j <= nBoth;
        const uint4 *sBb = sB[buf] + boff0;          // this lane's row n of the stage, tile 0
        const uint4 *sEb = sE[buf] + n;
#pragma unroll 1
        for (int tt = 0; tt < SC / 32; ++tt) {
            bf16x8_t b[NS];
#pragma unroll
            for (int kk = 0; kk < NK; ++kk) b[kk] = __builtin_bit_cast(bf16x8_t, sBb[tt * 32 * CH + bpiece[kk]]);
            b[NK] = __builtin_bit_cast(bf16x8_t, sEb[tt * 32]);
            float csum = 0.0f;
            if (j == 0) {
                // column tile index inside the block vs this wave's row tiles
                const int ctile = sin * (SC / 32) + tt;
                sym_tile<D, RTW, false, true>(a, b, racc, csum, s, n, hb, ctile - wave * RTW);
            } else if (both) {
                sym_tile<D, RTW, true, false>(a, b, racc, csum, s, n, hb, -1);
                // each half-wave keeps its own partial sum (no cross-lane step, no branch)
                csw[sin * SC + tt * 32] = csum;
            } else {
                sym_tile<D, RTW, false, false>(a, b, racc, csum, s, n, hb, -1);
            }
        }
        if (both && sin == SPB - 1) {
            __syncthreads();
            const int J = (I + j) % nB;
            unsigned long long *dst = acc + (size_t)h * Lpad + (size_t)J * BM;
            for (int c = tid; c < BM; c += 256)
                fixed_add(dst + c, ((cs[0][0][c] + cs[0][1][c]) + (cs[1][0][c] + cs[1][1][c])) +
                                       ((cs[2][0][c] + cs[2][1][c]) + (cs[3][0][c] + cs[3][1][c])));
        }
    }

    // each wave owns its rows: reduce over the 32 columns held by the lanes of a half-wave
#pragma unroll
    for (int rt = 0; rt < RTW; ++rt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float v = racc[rt][r];
            v += __shfl_xor(v, 1);
            v += __shfl_xor(v, 2);
            v += __shfl_xor(v, 4);
            v += __shfl_xor(v, 8);
            v += __shfl_xor(v, 16);
            if (n == 0)
                fixed_add(acc + (size_t)h * Lpad + I * BM + (wave * RTW + rt) * 32 + 8 * (r >> 2) + 4 * hb + (r & 3), v);
        }
}

// rho = accumulated kernel sum / L
__global__ void __launch_bounds__(256)
density_finish(const unsigned long long *__restrict__ acc, float *__restrict__ rho, int L, int Lpad, int head0)
{
    const int h = head0 + blockIdx.y;
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= L) return;
    const double t = (double)acc[(size_t)h * Lpad + i] * (1.0 / 4294967296.0);
    rho[(size_t)h * L + i] = (float)(t / (double)L);
}

// A launch of the symmetric sweep takes at most this many heads.
constexpr int kSymChunkHeads = 16384;

constexpr int kSymRtw64 = 2, kSymRtw128 = 2;   // row tiles per wave
static inline int sym_bm(int d) { return 128 * (d == 64 ? kSymRtw64 : kSymRtw128); }
static inline bool use_sym(bool bf16, int L, int d) { return bf16 && (L + sym_bm(d) - 1) / sym_bm(d) >= 4; }

// ------------------------------------------------------------------------------------------
struct DensityWs {
    size_t est, scale, kbase, cand, cvec, stat, nsum, ext, kc, acc, total;
    int Lpad, nB, nBoth;
};

static DensityWs density_layout(int H, int L, int d, bool bf16)
{
    DensityWs w;
    w.Lpad = density_lpad(L);
    size_t o = kDensityFlagBytes;                               // the flag block sits in front
    w.est = o;
    o += round_up((size_t)H * sizeof(float), 256);
    w.scale = o;
    o += round_up((size_t)H * sizeof(float), 256);
    w.kbase = o;
    o += round_up((size_t)H * sizeof(void *), 256);
    w.cand = o;
    o += round_up((size_t)H * sizeof(int), 256);
    w.cvec = o;
    o += round_up((size_t)H * d * sizeof(float), 256);
    w.stat = o;
    if (bf16) o += round_up((size_t)H * kStatChunks * 3 * d * sizeof(float), 256);
    w.nsum = o;
    o += round_up((size_t)H * (w.Lpad / 256) * sizeof(double), 256);
    w.ext = o;
    o += (size_t)H * w.Lpad * sizeof(uint4);
    w.kc = o;
    if (bf16) o += round_up((size_t)H * L * d * 2, 256);
    w.acc = o;
    w.nB = w.nBoth = 0;
    if (use_sym(bf16, L, d)) {
        w.nB = w.Lpad / sym_bm(d);
        w.nBoth = (w.nB - 1) / 2;
        o += round_up((size_t)H * w.Lpad * sizeof(unsigned long long), 256);
    }
    w.total = o;
    return w;
}

size_t density_workspace_bytes(int H, int L, int d, bool bf16) { return density_layout(H, L, d, bf16).total; }
size_t density_estimate_offset() { return kDensityFlagBytes; }

static PrepWs prep_pointers(const DensityWs &w, char *base)
{
    PrepWs p;
    p.flag = reinterpret_cast<int *>(base);
    p.est = reinterpret_cast<float *>(base + w.est);
    p.scale = reinterpret_cast<float *>(base + w.scale);
    p.kbase = reinterpret_cast<const void **>(base + w.kbase);
    p.cand = reinterpret_cast<int *>(base + w.cand);
    p.cvec = reinterpret_cast<float *>(base + w.cvec);
    p.stat = reinterpret_cast<float *>(base + w.stat);
    p.nsum = reinterpret_cast<double *>(base + w.nsum);
    p.ext = reinterpret_cast<uint4 *>(base + w.ext);
    p.Kc = base + w.kc;
    p.acc = w.nB ? reinterpret_cast<unsigned long long *>(base + w.acc) : nullptr;
    return p;
}

template <class TR, int D>
static void run_prep(const void *K, int H, int L, const float *sigma_host, const DensityWs &w, char *base,
                     hipStream_t st)
{
    typedef typename TR::Elem Elem;
    constexpr bool kBf16 = sizeof(Elem) == 2;
    const PrepWs p = prep_pointers(w, base);
    for (int pass = 0; pass < (kBf16 ? 2 : 1); ++pass) {
        if constexpr (kBf16) {
            for (int h0 = 0; h0 < H; h0 += 32768) {      // grid.y is 16 bits wide
                const int nh = (H - h0 < 32768) ? H - h0 : 32768;
                hipLaunchKernelGGL((density_stats<D>), dim3(kStatChunks, nh), dim3(256), 0, st,
                                   reinterpret_cast<const uint16_t *>(K) + (size_t)h0 * L * D,
                                   p.stat + (size_t)h0 * kStatChunks * 3 * D, L, pass, p.cand + h0);
            }
        }
        for (int h0 = 0; h0 < H; h0 += 256) {
            const int nh = (H - h0 < 256) ? H - h0 : 256;
            ScaleChunk sc;
            for (int i = 0; i < 256; ++i) {
                // exponent scale log2(e)/sigma^2, so the sweep can use the hardware exp2
                const double sg = (i < nh) ? (double)sigma_host[h0 + i] : 1.0;
                sc.s[i] = (float)(1.4426950408889634 / (sg * sg));
            }
            hipLaunchKernelGGL((density_decide<D>), dim3(nh), dim3(D), 0, st, p, K, (size_t)L * D * sizeof(Elem), sc, h0,
                               kBf16 ? 1 : 0);
        }
    }
    for (int h0 = 0; h0 < H; h0 += 32768) {      // grid.y is 16 bits wide
        const int nh = (H - h0 < 32768) ? H - h0 : 32768;
        PrepWs q = p;
        q.cvec += (size_t)h0 * D;
        q.kbase += h0;
        q.nsum += (size_t)h0 * (w.Lpad / 256);
        q.ext += (size_t)h0 * w.Lpad;
        q.Kc = reinterpret_cast<char *>(q.Kc) + (size_t)h0 * L * D * sizeof(Elem);
        if (q.acc) q.acc += (size_t)h0 * w.Lpad;
        hipLaunchKernelGGL((density_prep<TR, D>), dim3(w.Lpad / 256, nh), dim3(256), 0, st,
                           reinterpret_cast<const Elem *>(K) + (size_t)h0 * L * D, q, L, w.Lpad);
    }
    hipLaunchKernelGGL(density_estimate, dim3((H + 255) / 256), dim3(256), 0, st, p, H, L, w.Lpad);
}

template <class TR, int D, int RT>
static hipError_t run(const void *K, int H, int L, const float *sigma_host, float *rho, void *ws, hipStream_t st)
{
    typedef typename TR::Elem Elem;
    const DensityWs w = density_layout(H, L, D, sizeof(Elem) == 2);
    char *base = reinterpret_cast<char *>(ws);
    run_prep<TR, D>(K, H, L, sigma_host, w, base, st);
    const int BM = RT * 32;
    const int nRB = (L + BM - 1) / BM;
    const long long total = (long long)nRB * H;
    if (total > 0x7FFFFFFFLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL((density_sweep<TR, D, RT>), dim3((unsigned)total), dim3(256), 0, st,
                       reinterpret_cast<const void *const *>(base + w.kbase), reinterpret_cast<const uint4 *>(base + w.ext),
                       reinterpret_cast<const float *>(base + w.scale), rho, L, w.Lpad, nRB, (int)total);
    return hipGetLastError();
}

template <int D, int RTW>
static hipError_t run_sym(const void *K, int H, int L, const float *sigma_host, float *rho, void *ws, hipStream_t st)
{
    const DensityWs w = density_layout(H, L, D, true);
    char *base = reinterpret_cast<char *>(ws);
    run_prep<Bf16Tr, D>(K, H, L, sigma_host, w, base, st);
    unsigned long long *acc = reinterpret_cast<unsigned long long *>(base + w.acc);
    const int chunk = kSymChunkHeads;            // heads per launch (keeps the grid within 2^31 workgroups)
    for (int h0 = 0; h0 < H; h0 += chunk) {
        const int nh = (H - h0 < chunk) ? H - h0 : chunk;
        const int total = nh * w.nB;
        hipLaunchKernelGGL((density_sym<D, RTW>), dim3(total), dim3(256), 0, st,
                           reinterpret_cast<const void *const *>(base + w.kbase), reinterpret_cast<const uint4 *>(base + w.ext),
                           reinterpret_cast<const float *>(base + w.scale), acc, L, w.Lpad, w.nB, w.nBoth, h0, total);
        hipLaunchKernelGGL(density_finish, dim3((L + 255) / 256, nh), dim3(256), 0, st, acc, rho, L, w.Lpad, h0);
    }
    return hipGetLastError();
}

hipError_t launch_density(const void *K, bool bf16, int H, int L, int d, const float *sigma_host, float *rho,
                          void *ws, hipStream_t st)
{
    if (bf16) {
        if (use_sym(true, L, d)) {
            if (d == 64) return run_sym<64, kSymRtw64>(K, H, L, sigma_host, rho, ws, st);
            if (d == 128) return run_sym<128, kSymRtw128>(K, H, L, sigma_host, rho, ws, st);
        }
        if (d == 64) return run<Bf16Tr, 64, 4>(K, H, L, sigma_host, rho, ws, st);
        if (d == 128) return run<Bf16Tr, 128, 2>(K, H, L, sigma_host, rho, ws, st);
    } else {
        if (d == 64) return run<F32Tr, 64, 2>(K, H, L, sigma_host, rho, ws, st);
        if (d == 128) return run<F32Tr, 128, 1>(K, H, L, sigma_host, rho, ws, st);
    }
    return hipErrorInvalidValue;
}

// which sweep serves these sizes (for reports): 1 = symmetric, 0 = full
bool density_uses_symmetric(bool bf16, int L, int d) { return use_sym(bf16, L, d); }

}  // namespace ws
