// Stand-ins for the kernel launchers behind the C-ABI front end (csrc/api.hip), so that the front end's
// host-side validation can run inside a sanitizer build on a machine without a GPU.  Nothing here launches
// anything: a launcher that is reached records the call and reports success.
#include "../../paper_2601_01298_amd/csrc/ws_internal.h"

int g_launches = 0;

namespace ws {

size_t density_workspace_bytes(int H, int L, int, bool) { return (size_t)H * L * 16 + 256; }
size_t density_estimate_offset() { return kDensityFlagBytes; }
bool density_uses_symmetric(bool bf16, int L, int) { return bf16 && L >= 1024; }
hipError_t launch_density(const void *, bool, int, int, int, const float *, float *, void *, hipStream_t)
{
    ++g_launches;
    return hipSuccess;
}
Chip current_chip() { return Chip{256, 2}; }
size_t select_workspace_bytes(int H, int L, int, bool) { return kSelectFlagBytes + (size_t)H * L * 8; }
bool choose_select(int which, bool bf16, int, int L, int, const Chip &, size_t, SelectChoice &c)
{
    c.resident = bf16 && which != 1 && L <= 65536;
    if (!c.resident && L > 1000000) return false;      // as if not even one head's slabs fitted a budget
    c.stream = SelectPlan{8, 4, 512};
    c.res = ResidentShape{2, 0, 8, 16, 1};
    return !(which == 2 && !c.resident);
}
size_t stream_select_workspace_bytes(const SelectPlan &p, int L) { return kSelectFlagBytes + (size_t)p.groups * L * 8; }
size_t resident_select_workspace_bytes(int H) { return kSelectFlagBytes + (size_t)H * 1024; }
hipError_t select_static_scratch(void **) { return hipErrorNoDevice; }
hipError_t launch_select(const SelectChoice &, const void *, bool, int, int, int, const float *, int, float, int32_t *,
                         float *, void *, hipStream_t)
{
    ++g_launches;
    return hipSuccess;
}
hipError_t launch_gather(const void *, const void *, int, int, int, const int32_t *, int, void *, void *, hipStream_t)
{
    ++g_launches;
    return hipSuccess;
}
size_t attend_workspace_bytes(bool bf16, int N, int Hq, int Hkv, int k, int d)
{
    return (bf16 && Hkv <= 8 && k >= 2048) ? (size_t)4 * N * Hq * (d + 4) * 4 : 0;
}
hipError_t launch_attend(const void *, const void *, const void *, bool, int, int, int, int, int, float, float *, void *,
                         hipStream_t)
{
    ++g_launches;
    return hipSuccess;
}
hipError_t launch_attend_indexed(const void *, const void *, const void *, const int32_t *, bool, int, int, int, int, int,
                                 int, float, float *, void *, hipStream_t)
{
    ++g_launches;
    return hipSuccess;
}
bool mass_supported(int Hkv, int Hq) { return Hq <= 128 && Hq / Hkv <= 8; }
size_t mass_workspace_bytes(int, int Hq, int L) { return (size_t)Hq * L * 4; }
hipError_t launch_attention_mass(const void *, const void *, bool, int, int, int, int, int, float, int, float *, void *,
                                 hipStream_t)
{
    ++g_launches;
    return hipSuccess;
}
int append_max_rows() { return 32; }
size_t append_workspace_bytes(int H, int L) { return (size_t)H * L; }
hipError_t launch_density_append(const void *, bool, int, int, int, int, const float *, const float *, float *, void *,
                                 hipStream_t)
{
    ++g_launches;
    return hipSuccess;
}
hipError_t launch_gate(const void *, const void *, bool, int, int, float, float *, int32_t *, hipStream_t)
{
    ++g_launches;
    return hipSuccess;
}
size_t inject_workspace_bytes(int d, int m) { return (size_t)m * d * 4; }
hipError_t launch_inject(void *, void *, bool, int, int, int, int, const void *, const void *, int, const int32_t *, float,
                         void *, hipStream_t)
{
    ++g_launches;
    return hipSuccess;
}

}  // namespace ws
