// Internal declarations shared by the kernel files and the C-ABI front end.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace ws {

constexpr int kWave = 64;

static inline size_t round_up(size_t x, size_t m) { return (x + m - 1) / m * m; }

// fp32 -> bf16 bit pattern, round to nearest even (finite inputs)
__device__ __forceinline__ uint32_t bf16_rne(float f)
{
    const uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// Sum over aligned groups of LPR consecutive lanes (LPR a power of two); every lane of a group ends up with
// the group's sum.  Inside a row of 16 lanes the partners are reached by DPP operands of the add itself
// (swap in pairs, swap pairs in quads, mirror 8, mirror 16: the same partners as xor 1, 2, 4, 8, so the
// result is the xor butterfly's bit for bit); only wider groups go through the LDS crossbar.
template <int CTRL>
__device__ __forceinline__ float dpp_add_f32(float v)
{
    return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}

template <int LPR>
__device__ __forceinline__ float lane_group_sum(float v)
{
    if (LPR >= 2) v = dpp_add_f32<0xB1>(v);      // quad_perm [1,0,3,2]
    if (LPR >= 4) v = dpp_add_f32<0x4E>(v);      // quad_perm [2,3,0,1]
    if (LPR >= 8) v = dpp_add_f32<0x141>(v);     // row_half_mirror
    if (LPR >= 16) v = dpp_add_f32<0x140>(v);    // row_mirror
    if (LPR >= 32) v += __shfl_xor(v, 16);
    if (LPR >= 64) v += __shfl_xor(v, 32);
    return v;
}

// ---- density -------------------------------------------------------------------------
// Keys per head are padded to a multiple of 512 in the per-key side records.
static inline int density_lpad(int L) { return (int)round_up((size_t)L, 512); }
constexpr size_t kDensityFlagBytes = 256;     // head of the density workspace: int32 accuracy flag at offset 0
size_t density_workspace_bytes(int H, int L, int d, bool bf16);
size_t density_estimate_offset();             // where the per-head error estimates start (H floats)
bool density_uses_symmetric(bool bf16, int L, int d);
// sigma_host[h] > 0 (validated by the caller); enqueues prepass + main sweep.
hipError_t launch_density(const void *K, bool bf16, int H, int L, int d, const float *sigma_host,
                          float *rho, void *ws, hipStream_t st);

// ---- selection -----------------------------------------------------------------------
// What the selection kernels need to know about the chip they run on.  Both are persistent and their
// workgroups wait on each other, so a launch may never hold more workgroups than the device keeps
// resident at once: compute units x workgroups per unit.
struct Chip {
    int cus;         // compute units of the device
    int wg_per_cu;   // workgroups per compute unit; 0 = ask the runtime for the kernel instance in question
};
// The current device, or the MI355X figure (256 compute units) where no device is visible.
Chip current_chip();

constexpr size_t kSelectFlagBytes = 256;    // head of every selection workspace: int32 failure flag at offset 0
constexpr int kMaxResidentGroups = 1024;    // heads in flight the resident kernel's workspace is sized for
constexpr int kMaxStreamGroups = 32;        // heads in flight of the streaming kernel

struct SelectPlan {
    int groups;   // heads processed concurrently (each by `members` workgroups)
    int members;  // workgroups cooperating on one head
    int threads;  // threads per workgroup
};
// slab_budget: bytes the per-head distance and inverse-density slabs may take together (0 = no limit)
SelectPlan select_plan(int H, int L, const Chip &chip, size_t slab_budget);
size_t stream_select_workspace_bytes(const SelectPlan &p, int L);
size_t select_workspace_bytes(int H, int L, int d, bool bf16);

struct ResidentShape {
    int rreg, rlds;   // key rows per lane in registers and in LDS
    int wgpg;         // workgroups per head
    int groups;       // heads in flight
    int rounds;       // passes over the heads
};
// register/LDS-resident variant (bf16, heads small enough to sit on chip); false when no instance fits
bool resident_select_shape(int H, int L, int d, const Chip &chip, ResidentShape &shape);
size_t resident_select_workspace_bytes(int H);
hipError_t launch_select_resident(const void *K, int H, int L, int d, const float *rho, int k, float alpha,
                                  int32_t *idx, float *score_out, void *ws, const ResidentShape &shape, hipStream_t st);
// the same kernel with the next step's screen run during the exchange; d = 64 and eight rows per lane only,
// called by launch_select_resident with the workspace laid out and cleared
hipError_t launch_select_resident_ahead(const void *K, int H, int L, const float *rho, int k, float alpha, int32_t *idx,
                                        float *score_out, unsigned long long *slots, int *fail, int groups, int wgpg,
                                        hipStream_t st);
hipError_t resident_ahead_occupancy(int *workgroups_per_cu);

// which: 0 = the library chooses, 1 = streaming kernel, 2 = resident kernel
struct SelectChoice {
    bool resident;
    SelectPlan stream;
    ResidentShape res;
};
// false when `which` asks for the resident kernel and no instance fits these sizes on this chip
bool choose_select(int which, bool bf16, int H, int L, int d, const Chip &chip, size_t slab_budget, SelectChoice &c);
hipError_t launch_select(const SelectChoice &c, const void *K, bool bf16, int H, int L, int d, const float *rho, int k,
                         float alpha, int32_t *idx, float *score_out, void *ws, hipStream_t st);
// The no-allocation variant's scratch: a fixed array in device memory, one copy per device.
constexpr size_t kStaticSlabBytes = (size_t)4 << 20;       // distance + inverse-density slabs of the streaming kernel
constexpr size_t kStaticScratchBytes = kSelectFlagBytes + ((size_t)1 << 20) + kStaticSlabBytes;
hipError_t select_static_scratch(void **ptr);              // address of the current device's copy

// ---- gather --------------------------------------------------------------------------
hipError_t launch_gather(const void *K, const void *V, int row_bytes, int H, int L,
                         const int32_t *idx, int k, void *Ks, void *Vs, hipStream_t st);

// ---- attention -----------------------------------------------------------------------
// partial rows of a split landmark range (0 when the range is not split)
size_t attend_workspace_bytes(bool bf16, int N, int Hq, int Hkv, int k, int d);
hipError_t launch_attend(const void *Q, const void *Ks, const void *Vs, bool bf16, int N, int Hq,
                         int Hkv, int k, int d, float scale, float *O, void *ws, hipStream_t st);
// the same over rows idx[h,t] of the whole cache K, V [Hkv, L, d] (same workspace, bit-identical result)
hipError_t launch_attend_indexed(const void *Q, const void *K, const void *V, const int32_t *idx, bool bf16, int N,
                                 int Hq, int Hkv, int L, int k, int d, float scale, float *O, void *ws, hipStream_t st);

// ---- steps next to the hot path -------------------------------------------------------
bool mass_supported(int Hkv, int Hq);
size_t mass_workspace_bytes(int G, int Hq, int L);
hipError_t launch_attention_mass(const void *K, const void *Q, bool bf16, int G, int Hkv, int Hq, int L, int d,
                                 float scale, int as_density, float *out, void *ws, hipStream_t st);

int append_max_rows();
size_t append_workspace_bytes(int H, int L);
hipError_t launch_density_append(const void *K, bool bf16, int H, int L, int d, int m, const float *sigma_host,
                                 const float *rho_old, float *rho_new, void *ws, hipStream_t st);

hipError_t launch_gate(const void *hmain, const void *T, bool bf16, int N, int dm, float theta, float *score,
                       int32_t *accept, hipStream_t st);

size_t inject_workspace_bytes(int d, int m);
hipError_t launch_inject(void *Kc, void *Vc, bool bf16, int H, int Lcap, int d, int L, const void *Knew,
                         const void *Vnew, int m, const int32_t *pos, float base, void *ws, hipStream_t st);

// Workgroup ids are handed to the 8 accelerator dies (XCDs) round-robin, and each die has
// its own L2.  This maps a hardware workgroup id to a logical id so that each die works on
// one contiguous range of logical ids (neighbouring tiles of the same head share an L2).
__device__ __forceinline__ int xcd_contiguous(int b, int total)
{
    const int xcd = b & 7, j = b >> 3;
    const int per = total >> 3, rem = total & 7;
    const int start = (xcd < rem) ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per;
    return start + j;
}

}  // namespace ws
