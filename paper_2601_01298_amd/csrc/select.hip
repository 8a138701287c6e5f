// Greedy landmark selection by the hybrid coverage / inverse-density score (Warp-Cortex
// Sec. 3.3, "Hybrid Density-Coverage Sampler"; Sec. 2 first paragraph).  Per head, k dependent
// steps; step t
//   (1) folds the previous landmark into D_i = distance of key i to its nearest landmark
//       (direct coordinate differences in fp32, square root taken per key),
//   (2) finds D_max over the keys not yet chosen,
//   (3) scores  alpha * D_i / D_max + (1 - alpha) * u_i  and takes the argmax, lowest index on ties.
// One new landmark per step makes (1) a matrix-vector sweep over all keys of the head: the stage
// is bound by how fast key rows reach the vector ALUs, not by arithmetic.
//
// Streaming kernel (any L, any d in {64,128}): a head is owned by a GROUP of `members`
// workgroups that live on the same accelerator die (so they share its L2) and each own a
// contiguous slice of the keys.  The kernel is persistent: a group walks through its heads, and
// inside a head through the k steps; per step the members exchange one 64-bit word twice
// (their local D_max, then their local best candidate) through a small slot array in global
// memory.  Every word carries an 8-bit sequence tag, slots are double-buffered by exchange
// parity, and every wait is bounded: if it expires the group flags the failure, writes -1 into
// the index entries it still owes and leaves, so the grid always drains.
#include <atomic>

#include "ws_internal.h"

namespace ws {

namespace {

constexpr int kMaxMembers = 64;
constexpr unsigned kSpinLimit = 1u << 22;   // polls, a fraction of a microsecond apart: seconds in total

struct SelArgs {
    const void *K;
    const float *rho;
    int32_t *idx;
    float *score_out;
    float *Dws;                      // [groups][Lslab] distance to nearest landmark; -1 = chosen
    float *Uws;                      // [groups][Lslab] inverse density u_i
    unsigned long long *slots;       // [groups][2][kMaxMembers]
    int *fail;                       // set to 1 if a bounded wait expired
    int H, L, k, Lslab;
    int groups, members, slice;      // slice = keys per member (multiple of 64)
    float alpha;
};

__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long v)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        const unsigned long long w = __shfl_xor(v, o);
        v = (w > v) ? w : v;
    }
    return v;
}

// Order-preserving packing of a candidate: larger score wins, then lower index.
// Scores are >= 0, so their IEEE bit patterns order like unsigned integers.
__device__ __forceinline__ unsigned long long pack_cand(float score, int i)
{
    return ((unsigned long long)__float_as_uint(score) << 32) | ((unsigned long long)(0xFFFFFFu - (unsigned)i) << 8);
}

struct Block {
    unsigned long long red[16];
    unsigned long long result;
    int abort;
};

// Workgroup-wide max of a 64-bit word (low 8 bits must be 0), then group-wide through the slots.
// Returns the maximum over all members; every thread gets the same value.
template <int TPB>
__device__ __forceinline__ unsigned long long
group_max(unsigned long long v, Block &sh, const SelArgs &a, int group, int member, unsigned &seq)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    v = wave_max_u64(v);
    if (lane == 0) sh.red[wave] = v;
    __syncthreads();
    if (wave == 0) {
        unsigned long long w = (lane < TPB / 64) ? sh.red[lane] : 0ull;
        w = wave_max_u64(w);
        if (a.members > 1) {
            ++seq;
            const unsigned long long tag = (unsigned long long)(seq % 255u + 1u);
            unsigned long long *slot = a.slots + ((size_t)group * 2 + (seq & 1u)) * kMaxMembers;
            if (lane == 0)
                __hip_atomic_store(slot + member, w | tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            bool ok = lane >= a.members;
            unsigned long long got = 0ull;
            unsigned spins = 0;
            while (true) {
                if (!ok) {
                    got = __hip_atomic_load(slot + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    ok = (got & 0xFFull) == tag;
                }
                if (__all(ok)) break;
                if (++spins > kSpinLimit) break;
                if (spins > 64) __builtin_amdgcn_s_sleep(8);
            }
            if (!__all(ok)) {
                if (lane == 0) {
                    sh.abort = 1;
                    atomicExch(a.fail, 1);
                }
                got = 0ull;
            }
            w = wave_max_u64(ok && lane < a.members ? (got & ~0xFFull) : 0ull);
        }
        if (lane == 0) sh.result = w;
    }
    __syncthreads();
    return sh.result;
}

template <typename T> struct Row;
template <> struct Row<uint16_t> {   // bf16: 8 elements per 16-byte chunk
    static constexpr int PER = 8;
    static __device__ __forceinline__ void unpack(const uint4 &q, float *f)
    {
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(w[i] << 16);
            f[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
        }
    }
};
template <> struct Row<float> {      // fp32: 4 elements per 16-byte chunk
    static constexpr int PER = 4;
    static __device__ __forceinline__ void unpack(const uint4 &q, float *f)
    {
        f[0] = __uint_as_float(q.x);
        f[1] = __uint_as_float(q.y);
        f[2] = __uint_as_float(q.z);
        f[3] = __uint_as_float(q.w);
    }
};

template <typename T, int D, int TPB>
__global__ void __launch_bounds__(TPB)
select_stream(SelArgs a)
{
    constexpr int PER = Row<T>::PER;
    constexpr int LPR = D / PER;          // lanes cooperating on one key row (8, 16 or 32)
    constexpr int RPI = TPB / LPR;        // rows per sweep iteration of the workgroup
    __shared__ Block sh;

    // group = set of workgroups on one die when the grid divides evenly over the 8 dies
    int group, member;
    if ((a.groups & 7) == 0) {
        const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
        group = xcd * (a.groups >> 3) + j / a.members;
        member = j % a.members;
    } else {
        group = blockIdx.x / a.members;
        member = blockIdx.x % a.members;
    }
    if (threadIdx.x == 0) sh.abort = 0;
    __syncthreads();

    const int sub = threadIdx.x % LPR;                 // which 16-byte chunk of a row
    const int rsub = threadIdx.x / LPR;                // which row of the iteration
    const int lo = member * a.slice;
    const int hi = min(a.L, lo + a.slice);
    float *Dg = a.Dws + (size_t)group * a.Lslab;
    float *Ug = a.Uws + (size_t)group * a.Lslab;
    const float alpha = a.alpha, oma = 1.0f - a.alpha;
    unsigned seq = 0;

    for (int h = group; h < a.H; h += a.groups) {
        const T *Kh = reinterpret_cast<const T *>(a.K) + (size_t)h * a.L * D;
        const float *rhoh = a.rho + (size_t)h * a.L;
        int t = 0;

        // ---- head set-up: rho_min over the head, u_i = rho_min / rho_i, D_i = +inf
        float rmin = __builtin_inff();
        for (int i = lo + (int)threadIdx.x; i < hi; i += TPB) rmin = fminf(rmin, rhoh[i]);
        // min over positive floats = max over the complemented bit pattern
        unsigned long long w = (unsigned long long)(0xFFFFFFFFu - __float_as_uint(rmin)) << 32;
        w = group_max<TPB>(w, sh, a, group, member, seq);
        if (sh.abort) goto bail;
        rmin = __uint_as_float(0xFFFFFFFFu - (unsigned)(w >> 32));
        for (int i = lo + (int)threadIdx.x; i < hi; i += TPB) {
            Ug[i] = rmin / rhoh[i];
            Dg[i] = __builtin_inff();
        }
        __syncthreads();

        {
            int prev = -1;
            for (t = 0; t < a.k; ++t) {
                float dmax = 0.0f;
                if (t > 0) {
                    // ---- (1)+(2): fold landmark `prev` into D, local max of D over unchosen keys
                    float lm[PER];
                    Row<T>::unpack(*reinterpret_cast<const uint4 *>(Kh + (size_t)prev * D + sub * PER), lm);
                    float lmax = 0.0f;
                    constexpr int UN = 4;      // key rows in flight per lane: the sweep is latency-bound otherwise
                    for (int r0 = lo; r0 < hi; r0 += UN * RPI) {
                        uint4 q[UN];
                        float dold[UN];
#pragma unroll
                        for (int u = 0; u < UN; ++u) {
                            const int i = r0 + u * RPI + rsub;
                            const int ic = min(i, hi - 1);
                            q[u] = *reinterpret_cast<const uint4 *>(Kh + (size_t)ic * D + sub * PER);
                            dold[u] = (sub == 0) ? Dg[ic] : 0.0f;
                        }
#pragma unroll
                        for (int u = 0; u < UN; ++u) {
                            const int i = r0 + u * RPI + rsub;
                            float f[PER];
                            Row<T>::unpack(q[u], f);
                            float acc = 0.0f;
#pragma unroll
                            for (int c = 0; c < PER; ++c) {
                                const float df = f[c] - lm[c];
                                acc = fmaf(df, df, acc);
                            }
#pragma unroll
                            for (int o = 1; o < LPR; o <<= 1) acc += __shfl_xor(acc, o);
                            if (sub == 0 && i < hi && dold[u] >= 0.0f) {
                                const float dist = __fsqrt_rn(acc);
                                float dn = dold[u];
                                if (dist < dn) {
                                    dn = dist;
                                    Dg[i] = dist;
                                }
                                lmax = fmaxf(lmax, dn);
                            }
                        }
                    }
                    __syncthreads();   // D of this slice is complete before it is scored
                    const unsigned long long wm =
                        group_max<TPB>((unsigned long long)__float_as_uint(lmax) << 32, sh, a, group, member, seq);
                    if (sh.abort) goto bail;
                    dmax = __uint_as_float((unsigned)(wm >> 32));
                }

                int s;
                float sc;
                if (t == 0 && alpha == 1.0f) {
                    s = 0;
                    sc = alpha;
                } else {
                    // ---- (3): score and argmax over unchosen keys
                    unsigned long long best = 0ull;
                    for (int i = lo + (int)threadIdx.x; i < hi; i += TPB) {
                        const float di = Dg[i];
                        if (di >= 0.0f) {
                            const float c = (t == 0) ? 1.0f : (dmax > 0.0f ? di / dmax : 0.0f);
                            const float v = alpha * c + oma * Ug[i];
                            const unsigned long long cand = pack_cand(v, i);
                            best = cand > best ? cand : best;
                        }
                    }
                    best = group_max<TPB>(best, sh, a, group, member, seq);
                    if (sh.abort) goto bail;
                    s = min((int)(0xFFFFFFu - (unsigned)((best >> 8) & 0xFFFFFFull)), a.L - 1);   // in range whatever the inputs held
                    sc = __uint_as_float((unsigned)(best >> 32));
                }
                if (member == 0 && threadIdx.x == 0) {
                    a.idx[(size_t)h * a.k + t] = s;
                    if (a.score_out) a.score_out[(size_t)h * a.k + t] = sc;
                }
                if (threadIdx.x == 0 && s >= lo && s < hi) Dg[s] = -1.0f;   // chosen: never scored again
                __syncthreads();
                prev = s;
            }
        }
        continue;
    bail:
        // a wait expired: mark what this group still owes as invalid and leave
        if (member == 0) {
            for (int hh = h; hh < a.H; hh += a.groups) {
                const int t0 = (hh == h) ? t : 0;
                for (int tt = t0 + (int)threadIdx.x; tt < a.k; tt += TPB) a.idx[(size_t)hh * a.k + tt] = -1;
            }
        }
        return;
    }
}

__global__ void select_clear(unsigned long long *slots, int n, int *fail)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) slots[i] = 0ull;
    if (i == 0) *fail = 0;
}

struct WsLayout {
    size_t slots, D, U, total;
    int Lslab;
};

WsLayout layout(const SelectPlan &p, int L)
{
    WsLayout w;
    w.Lslab = (int)round_up((size_t)L, 64);
    w.slots = kSelectFlagBytes;       // the failure flag sits in front
    w.D = w.slots + round_up((size_t)p.groups * 2 * kMaxMembers * sizeof(unsigned long long), 256);
    w.U = w.D + round_up((size_t)p.groups * w.Lslab * sizeof(float), 256);
    w.total = w.U + round_up((size_t)p.groups * w.Lslab * sizeof(float), 256);
    return w;
}

template <typename T, int D>
hipError_t run_select(const SelArgs &a, const SelectPlan &p, hipStream_t st)
{
    hipLaunchKernelGGL((select_stream<T, D, 512>), dim3(p.groups * p.members), dim3(512), 0, st, a);
    return hipGetLastError();
}

// Workgroups of the streaming kernel a compute unit holds at once (two where there is no device to ask).
int stream_occupancy()
{
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, select_stream<uint16_t, 128, 512>, 512, 0) != hipSuccess) {
        (void)hipGetLastError();
        return 2;
    }
    return n < 2 ? n : 2;       // the launch shapes are tuned for two; the answer guards against fewer
}

// Scratch of the entry point that allocates nothing.  In host code this name is only a handle: the
// address of a device's copy comes from hipGetSymbolAddress, once per device.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::atomic<void *> scratch_of_device[kMaxDevices];

}  // namespace

hipError_t select_static_scratch(void **ptr)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    void *p = scratch_of_device[dev].load(std::memory_order_acquire);
    if (p == nullptr) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (p == nullptr) return hipErrorInvalidSymbol;
        scratch_of_device[dev].store(p, std::memory_order_release);     // every thread would store the same address
    }
    *ptr = p;
    return hipSuccess;
}

Chip current_chip()
{
    Chip c{256, 0};
    int dev = -1, cus = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
        c.cus = cus;
    else
        (void)hipGetLastError();
    return c;
}

// How a launch of the streaming kernel is shaped.  A group's members wait on each other, so the whole
// grid must be resident at once: groups * members never exceeds compute units x workgroups per unit.
// Few heads -> many members per head; many heads -> the heads are walked through in rounds.
SelectPlan select_plan(int H, int L, const Chip &chip, size_t slab_budget)
{
    SelectPlan p;
    p.threads = 512;
    const int occ = chip.wg_per_cu > 0 ? chip.wg_per_cu : stream_occupancy();
    long long max_wg = (long long)chip.cus * occ;
    if (max_wg < 1) max_wg = 1;
    int groups = H < kMaxStreamGroups ? H : kMaxStreamGroups;
    if (groups > max_wg) groups = (int)max_wg;
    if (slab_budget > 0) {
        const size_t per_group = 2 * round_up(round_up((size_t)L, 64) * sizeof(float), 256);
        const size_t fit = slab_budget / per_group;
        if (fit < (size_t)groups) groups = (int)fit;       // 0: the slabs of one head do not fit
    }
    if (groups >= 8) groups -= groups % 8;
    int m2 = 1;
    if (groups > 0) {
        const long long members = max_wg / groups;
        while (m2 * 2 <= members && m2 * 2 <= kMaxMembers) m2 *= 2;
        // no point in slices smaller than one sweep iteration per member
        while (m2 > 1 && (L + m2 - 1) / m2 < 256) m2 /= 2;
    }
    p.groups = groups;
    p.members = m2;
    return p;
}

size_t stream_select_workspace_bytes(const SelectPlan &p, int L) { return layout(p, L).total; }

size_t select_workspace_bytes(int H, int L, int d, bool bf16)
{
    // Large enough for either kernel on any chip, so that the size does not depend on the device that
    // happens to be current when it is asked for: the streaming kernel at its largest number of heads in
    // flight, the resident one with a slot block for every head.
    (void)d;
    SelectPlan p;
    p.groups = H < kMaxStreamGroups ? H : kMaxStreamGroups;
    p.members = 1;
    p.threads = 512;
    size_t n = layout(p, L).total;
    if (bf16) {
        const size_t r = resident_select_workspace_bytes(H);
        if (r > n) n = r;
    }
    return n;
}

bool choose_select(int which, bool bf16, int H, int L, int d, const Chip &chip, size_t slab_budget, SelectChoice &c)
{
    c.resident = false;
    c.res = ResidentShape{0, 0, 0, 0, 0};
    c.stream = SelectPlan{0, 0, 0};
    const bool can_res = bf16 && which != 1 && resident_select_shape(H, L, d, chip, c.res);
    if (which == 2 && !can_res) return false;
    c.resident = can_res;
    if (!c.resident) {
        c.stream = select_plan(H, L, chip, slab_budget);
        if (c.stream.groups < 1) return false;
    }
    return true;
}

hipError_t launch_select(const SelectChoice &c, const void *K, bool bf16, int H, int L, int d, const float *rho, int k,
                         float alpha, int32_t *idx, float *score_out, void *ws, hipStream_t st)
{
    if (c.resident) return launch_select_resident(K, H, L, d, rho, k, alpha, idx, score_out, ws, c.res, st);

    const SelectPlan &p = c.stream;
    const WsLayout w = layout(p, L);
    char *base = reinterpret_cast<char *>(ws);
    SelArgs a;
    a.K = K;
    a.rho = rho;
    a.idx = idx;
    a.score_out = score_out;
    a.fail = reinterpret_cast<int *>(base);
    a.slots = reinterpret_cast<unsigned long long *>(base + w.slots);
    a.Dws = reinterpret_cast<float *>(base + w.D);
    a.Uws = reinterpret_cast<float *>(base + w.U);
    a.H = H;
    a.L = L;
    a.k = k;
    a.Lslab = w.Lslab;
    a.groups = p.groups;
    a.members = p.members;
    a.slice = (int)round_up((size_t)(L + p.members - 1) / p.members, 64);
    a.alpha = alpha;
    const int nslots = p.groups * 2 * kMaxMembers;
    hipLaunchKernelGGL(select_clear, dim3((nslots + 255) / 256), dim3(256), 0, st, a.slots, nslots, a.fail);
    if (bf16) {
        if (d == 64) return run_select<uint16_t, 64>(a, p, st);
        if (d == 128) return run_select<uint16_t, 128>(a, p, st);
    } else {
        if (d == 64) return run_select<float, 64>(a, p, st);
        if (d == 128) return run_select<float, 128>(a, p, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace ws
