// C-ABI front end: argument validation on the host, then the kernel launchers.
// Nothing here allocates, synchronises the host or keeps state between calls.
#include "../../include/ws_synapse.h"

#include <cmath>

#include "ws_internal.h"

namespace {

bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

ws_status check_common(ws_dtype dt, int d)
{
    if (dt != WS_F32 && dt != WS_BF16) return WS_ERR_UNSUPPORTED;
    if (d != 64 && d != 128) return WS_ERR_UNSUPPORTED;
    return WS_OK;
}

ws_status check_ws(const void *ws, size_t have, size_t need)
{
    if (need == 0) return WS_OK;
    if (ws == nullptr || !aligned(ws, 256) || have < need) return WS_ERR_WORKSPACE;
    return WS_OK;
}

constexpr int kMaxL = 1 << 24;   // candidate indices travel in 24 bits inside the selection kernel

}  // namespace

extern "C" {

size_t ws_synapse_workspace_bytes(ws_op op, ws_dtype dt, int H, int L, int d, int k, int N, int Hq)
{
    if (check_common(dt, d) != WS_OK) return (size_t)-1;
    switch (op) {
    case WS_OP_DENSITY:
        if (H < 1 || L < 1 || L >= kMaxL) return (size_t)-1;
        return ws::density_workspace_bytes(H, L, d, dt == WS_BF16);
    case WS_OP_SELECT:
        if (H < 1 || L < 1 || L >= kMaxL) return (size_t)-1;
        return ws::select_workspace_bytes(H, L, d, dt == WS_BF16);
    case WS_OP_GATHER:
        return 0;
    case WS_OP_ATTEND:
        // H = KV heads, Hq = query heads, L is not used
        if (H < 1 || Hq < 1 || N < 1 || k < 1 || Hq % H != 0) return (size_t)-1;
        return ws::attend_workspace_bytes(dt == WS_BF16, N, Hq, H, k, d);
    case WS_OP_ATTENTION_MASS:
        // H = KV heads in all groups, Hq = query heads in all groups: per-head logits and tile partials
        if (H < 1 || Hq < 1 || L < 1 || L >= kMaxL) return (size_t)-1;
        return ws::mass_workspace_bytes(1, Hq, L);
    case WS_OP_DENSITY_APPEND:
        if (H < 1 || L < 1 || L >= kMaxL) return (size_t)-1;
        return ws::append_workspace_bytes(H, L);
    case WS_OP_INJECT:
        if (k < 1) return (size_t)-1;
        return ws::inject_workspace_bytes(d, k);
    case WS_OP_INT_RANGE: break;
    }
    return (size_t)-1;
}

ws_status ws_synapse_density(const void *K, ws_dtype dt, int H, int L, int d, const float *sigma_host, float *rho,
                             void *workspace, size_t workspace_bytes, ws_stream stream)
{
    ws_status s = check_common(dt, d);
    if (s != WS_OK) return s;
    if (!K || !sigma_host || !rho || H < 1 || L < 1) return WS_ERR_INVALID_ARG;
    if (L >= kMaxL) return WS_ERR_UNSUPPORTED;
    if (!aligned(K, 16) || !aligned(rho, 4)) return WS_ERR_INVALID_ARG;
    s = check_ws(workspace, workspace_bytes, ws::density_workspace_bytes(H, L, d, dt == WS_BF16));
    if (s != WS_OK) return s;
    for (int h = 0; h < H; ++h) {
        const double sg = (double)sigma_host[h];
        const float sc = (float)(1.4426950408889634 / (sg * sg));   // the exponent scale the kernel will use
        if (!(sg > 0.0) || !std::isfinite(sg) || !std::isfinite(sc) || sc <= 0.0f) return WS_ERR_INVALID_ARG;
        // padded key slots carry -1e30 in place of -|k|^2/2: their kernel value must underflow to exactly 0
        if (sc * 1.0e30f < 256.0f) return WS_ERR_UNSUPPORTED;
    }
    const hipError_t e = ws::launch_density(K, dt == WS_BF16, H, L, d, sigma_host, rho, workspace, (hipStream_t)stream);
    return e == hipSuccess ? WS_OK : WS_ERR_HIP;
}

ws_status ws_synapse_density_check(const void *workspace, int H, ws_stream stream, int *flagged, float *err_est)
{
    if (!workspace || H < 1 || !flagged) return WS_ERR_INVALID_ARG;
    int flag = 0;
    const char *base = reinterpret_cast<const char *>(workspace);
    if (hipMemcpyAsync(&flag, base, sizeof(int), hipMemcpyDeviceToHost, (hipStream_t)stream) != hipSuccess) return WS_ERR_HIP;
    if (err_est && hipMemcpyAsync(err_est, base + ws::density_estimate_offset(), (size_t)H * sizeof(float),
                                  hipMemcpyDeviceToHost, (hipStream_t)stream) != hipSuccess)
        return WS_ERR_HIP;
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return WS_ERR_HIP;
    *flagged = flag != 0;
    return WS_OK;
}

namespace {

ws_status check_select_args(const void *K, ws_dtype dt, int H, int L, int d, const float *rho, int k, float alpha,
                            const int32_t *idx)
{
    ws_status s = check_common(dt, d);
    if (s != WS_OK) return s;
    if (!K || !rho || !idx || H < 1 || L < 1 || k < 1 || k > L) return WS_ERR_INVALID_ARG;
    if (!(alpha >= 0.0f && alpha <= 1.0f)) return WS_ERR_INVALID_ARG;
    if (L >= kMaxL) return WS_ERR_UNSUPPORTED;
    if (!aligned(K, 16) || !aligned(rho, 4) || !aligned(idx, 4)) return WS_ERR_INVALID_ARG;
    return WS_OK;
}

}  // namespace

ws_status ws_synapse_select_with(ws_select_kernel which, const void *K, ws_dtype dt, int H, int L, int d,
                                 const float *rho, int k, float alpha, int32_t *idx, float *score_out,
                                 void *workspace, size_t workspace_bytes, ws_stream stream)
{
    if (which != WS_SELECT_AUTO && which != WS_SELECT_STREAMING && which != WS_SELECT_RESIDENT) return WS_ERR_INVALID_ARG;
    ws_status s = check_select_args(K, dt, H, L, d, rho, k, alpha, idx);
    if (s != WS_OK) return s;
    s = check_ws(workspace, workspace_bytes, ws::select_workspace_bytes(H, L, d, dt == WS_BF16));
    if (s != WS_OK) return s;
    ws::SelectChoice c;
    if (!ws::choose_select((int)which, dt == WS_BF16, H, L, d, ws::current_chip(), 0, c)) return WS_ERR_UNSUPPORTED;
    const hipError_t e = ws::launch_select(c, K, dt == WS_BF16, H, L, d, rho, k, alpha, idx, score_out, workspace,
                                           (hipStream_t)stream);
    return e == hipSuccess ? WS_OK : WS_ERR_HIP;
}

ws_status ws_synapse_select(const void *K, ws_dtype dt, int H, int L, int d, const float *rho, int k, float alpha,
                            int32_t *idx, float *score_out, void *workspace, size_t workspace_bytes,
                            ws_stream stream)
{
    return ws_synapse_select_with(WS_SELECT_AUTO, K, dt, H, L, d, rho, k, alpha, idx, score_out, workspace,
                                  workspace_bytes, stream);
}

ws_status ws_synapse_select_static(const void *K, ws_dtype dt, int H, int L, int d, const float *rho, int k,
                                   float alpha, int32_t *idx, float *score_out, ws_stream stream)
{
    ws_status s = check_select_args(K, dt, H, L, d, rho, k, alpha, idx);
    if (s != WS_OK) return s;
    ws::SelectChoice c;
    if (!ws::choose_select(0, dt == WS_BF16, H, L, d, ws::current_chip(), ws::kStaticSlabBytes, c)) return WS_ERR_TOO_LARGE;
    const size_t need = c.resident ? ws::resident_select_workspace_bytes(c.res.groups)
                                   : ws::stream_select_workspace_bytes(c.stream, L);
    if (need > ws::kStaticScratchBytes) return WS_ERR_TOO_LARGE;
    void *scratch_ptr = nullptr;
    if (ws::select_static_scratch(&scratch_ptr) != hipSuccess) return WS_ERR_HIP;
    const hipError_t e = ws::launch_select(c, K, dt == WS_BF16, H, L, d, rho, k, alpha, idx, score_out, scratch_ptr,
                                           (hipStream_t)stream);
    return e == hipSuccess ? WS_OK : WS_ERR_HIP;
}

ws_status ws_synapse_select_failed(const void *workspace, ws_stream stream, int *failed)
{
    if (!failed) return WS_ERR_INVALID_ARG;
    const void *src = workspace;
    if (!src) {
        void *p = nullptr;
        if (ws::select_static_scratch(&p) != hipSuccess) return WS_ERR_HIP;
        src = p;
    }
    int flag = 0;
    if (hipMemcpyAsync(&flag, src, sizeof(int), hipMemcpyDeviceToHost, (hipStream_t)stream) != hipSuccess) return WS_ERR_HIP;
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return WS_ERR_HIP;
    *failed = flag != 0;
    return WS_OK;
}

ws_status ws_synapse_select_plan(ws_select_kernel which, ws_dtype dt, int H, int L, int d, int compute_units,
                                 int workgroups_per_cu, ws_select_plan *plan)
{
    if (which != WS_SELECT_AUTO && which != WS_SELECT_STREAMING && which != WS_SELECT_RESIDENT) return WS_ERR_INVALID_ARG;
    ws_status s = check_common(dt, d);
    if (s != WS_OK) return s;
    if (!plan || H < 1 || L < 1 || compute_units < 0 || workgroups_per_cu < 0) return WS_ERR_INVALID_ARG;
    if (L >= kMaxL) return WS_ERR_UNSUPPORTED;
    ws::Chip chip = ws::current_chip();
    if (compute_units > 0) chip.cus = compute_units;
    chip.wg_per_cu = workgroups_per_cu;
    ws::SelectChoice c;
    if (!ws::choose_select((int)which, dt == WS_BF16, H, L, d, chip, 0, c)) return WS_ERR_UNSUPPORTED;
    plan->resident = c.resident ? 1 : 0;
    plan->heads_in_flight = c.resident ? c.res.groups : c.stream.groups;
    plan->workgroups_per_head = c.resident ? c.res.wgpg : c.stream.members;
    plan->threads = c.resident ? 256 : c.stream.threads;
    plan->rows_in_registers = c.resident ? c.res.rreg : 0;
    plan->rows_in_lds = c.resident ? c.res.rlds : 0;
    plan->compute_units = chip.cus;
    return WS_OK;
}

ws_status ws_synapse_gather(const void *K, const void *V, ws_dtype dt, int H, int L, int d, const int32_t *idx, int k,
                            void *Ks, void *Vs, ws_stream stream)
{
    ws_status s = check_common(dt, d);
    if (s != WS_OK) return s;
    if (!K || !V || !idx || !Ks || !Vs || H < 1 || L < 1 || k < 1) return WS_ERR_INVALID_ARG;
    if (!aligned(K, 16) || !aligned(V, 16) || !aligned(Ks, 16) || !aligned(Vs, 16) || !aligned(idx, 4))
        return WS_ERR_INVALID_ARG;
    const int row_bytes = d * (dt == WS_BF16 ? 2 : 4);
    const hipError_t e = ws::launch_gather(K, V, row_bytes, H, L, idx, k, Ks, Vs, (hipStream_t)stream);
    return e == hipSuccess ? WS_OK : WS_ERR_HIP;
}

ws_status ws_synapse_attend(const void *Q, const void *Ks, const void *Vs, ws_dtype dt, int N, int Hq, int Hkv, int k,
                            int d, float scale, float *O, void *workspace, size_t workspace_bytes, ws_stream stream)
{
    ws_status s = check_common(dt, d);
    if (s != WS_OK) return s;
    if (!Q || !Ks || !Vs || !O || N < 1 || Hq < 1 || Hkv < 1 || k < 1) return WS_ERR_INVALID_ARG;
    if (Hq % Hkv != 0) return WS_ERR_INVALID_ARG;
    if (Hkv > 65535) return WS_ERR_UNSUPPORTED;
    if (!aligned(Q, 16) || !aligned(Ks, 16) || !aligned(Vs, 16) || !aligned(O, 16)) return WS_ERR_INVALID_ARG;
    if (!std::isfinite(scale)) return WS_ERR_INVALID_ARG;
    if (scale <= 0.0f) scale = 1.0f / std::sqrt((float)d);
    s = check_ws(workspace, workspace_bytes, ws::attend_workspace_bytes(dt == WS_BF16, N, Hq, Hkv, k, d));
    if (s != WS_OK) return s;
    const hipError_t e = ws::launch_attend(Q, Ks, Vs, dt == WS_BF16, N, Hq, Hkv, k, d, scale, O, workspace,
                                           (hipStream_t)stream);
    return e == hipSuccess ? WS_OK : WS_ERR_HIP;
}

ws_status ws_synapse_attend_indexed(const void *Q, const void *K, const void *V, const int32_t *idx, ws_dtype dt, int N,
                                    int Hq, int Hkv, int L, int k, int d, float scale, float *O, void *workspace,
                                    size_t workspace_bytes, ws_stream stream)
{
    ws_status s = check_common(dt, d);
    if (s != WS_OK) return s;
    if (!Q || !K || !V || !idx || !O || N < 1 || Hq < 1 || Hkv < 1 || L < 1 || k < 1) return WS_ERR_INVALID_ARG;
    if (Hq % Hkv != 0) return WS_ERR_INVALID_ARG;
    if (Hkv > 65535) return WS_ERR_UNSUPPORTED;
    if ((unsigned long long)L * d * (dt == WS_BF16 ? 2 : 4) >= (1ull << 32)) return WS_ERR_UNSUPPORTED;
    if (!aligned(Q, 16) || !aligned(K, 16) || !aligned(V, 16) || !aligned(O, 16) || !aligned(idx, 4))
        return WS_ERR_INVALID_ARG;
    if (!std::isfinite(scale)) return WS_ERR_INVALID_ARG;
    if (scale <= 0.0f) scale = 1.0f / std::sqrt((float)d);
    s = check_ws(workspace, workspace_bytes, ws::attend_workspace_bytes(dt == WS_BF16, N, Hq, Hkv, k, d));
    if (s != WS_OK) return s;
    const hipError_t e = ws::launch_attend_indexed(Q, K, V, idx, dt == WS_BF16, N, Hq, Hkv, L, k, d, scale, O, workspace,
                                                   (hipStream_t)stream);
    return e == hipSuccess ? WS_OK : WS_ERR_HIP;
}

ws_status ws_synapse_attention_mass(const void *K, const void *Q, ws_dtype dt, int G, int Hkv, int Hq, int L, int d,
                                    float scale, int as_density, float *out, void *workspace, size_t workspace_bytes,
                                    ws_stream stream)
{
    ws_status s = check_common(dt, d);
    if (s != WS_OK) return s;
    if (!K || !Q || !out || G < 1 || Hkv < 1 || Hq < 1 || L < 1 || Hq % Hkv != 0) return WS_ERR_INVALID_ARG;
    if (!std::isfinite(scale) || !aligned(K, 16) || !aligned(Q, 16) || !aligned(out, 4)) return WS_ERR_INVALID_ARG;
    if (L >= kMaxL || !ws::mass_supported(Hkv, Hq) || (long long)G * Hkv > 65535 || (long long)G * Hq > (1 << 20))
        return WS_ERR_UNSUPPORTED;
    if (G > 65535) return WS_ERR_UNSUPPORTED;
    s = check_ws(workspace, workspace_bytes, ws::mass_workspace_bytes(G, Hq, L));
    if (s != WS_OK) return s;
    if (scale <= 0.0f) scale = 1.0f / std::sqrt((float)d);
    const hipError_t e = ws::launch_attention_mass(K, Q, dt == WS_BF16, G, Hkv, Hq, L, d, scale, as_density, out,
                                                   workspace, (hipStream_t)stream);
    return e == hipSuccess ? WS_OK : WS_ERR_HIP;
}

ws_status ws_synapse_density_append(const void *K, ws_dtype dt, int H, int L, int d, int m, const float *sigma_host,
                                    const float *rho_old, float *rho_new, void *workspace, size_t workspace_bytes,
                                    ws_stream stream)
{
    ws_status s = check_common(dt, d);
    if (s != WS_OK) return s;
    if (!K || !sigma_host || !rho_old || !rho_new || H < 1 || L < 2 || m < 1 || m >= L) return WS_ERR_INVALID_ARG;
    if (L >= kMaxL || m > ws::append_max_rows()) return WS_ERR_UNSUPPORTED;
    if (!aligned(K, 16) || !aligned(rho_old, 4) || !aligned(rho_new, 4)) return WS_ERR_INVALID_ARG;
    s = check_ws(workspace, workspace_bytes, ws::append_workspace_bytes(H, L));
    if (s != WS_OK) return s;
    for (int h = 0; h < H; ++h) {
        const double sg = (double)sigma_host[h];
        const float sc = (float)(0.5 * 1.4426950408889634 / (sg * sg));
        if (!(sg > 0.0) || !std::isfinite(sg) || !std::isfinite(sc) || sc <= 0.0f) return WS_ERR_INVALID_ARG;
    }
    const hipError_t e = ws::launch_density_append(K, dt == WS_BF16, H, L, d, m, sigma_host, rho_old, rho_new,
                                                   workspace, (hipStream_t)stream);
    return e == hipSuccess ? WS_OK : WS_ERR_HIP;
}

ws_status ws_synapse_gate(const void *h_main, const void *T, ws_dtype dt, int N, int dm, float theta, float *score,
                          int32_t *accept, ws_stream stream)
{
    if (dt != WS_F32 && dt != WS_BF16) return WS_ERR_UNSUPPORTED;
    if (!h_main || !T || !score || !accept || N < 1 || dm < 1 || std::isnan(theta)) return WS_ERR_INVALID_ARG;
    const size_t es = dt == WS_BF16 ? 2 : 4;
    if (!aligned(h_main, es) || !aligned(T, es) || !aligned(score, 4) || !aligned(accept, 4)) return WS_ERR_INVALID_ARG;
    if (((long long)N + 3) / 4 > 0x7FFFFFFFLL) return WS_ERR_UNSUPPORTED;
    const hipError_t e = ws::launch_gate(h_main, T, dt == WS_BF16, N, dm, theta, score, accept, (hipStream_t)stream);
    return e == hipSuccess ? WS_OK : WS_ERR_HIP;
}

ws_status ws_synapse_inject(void *Kc, void *Vc, ws_dtype dt, int H, int Lcap, int d, int L, const void *Knew,
                            const void *Vnew, int m, const int32_t *pos, float base, void *workspace,
                            size_t workspace_bytes, ws_stream stream)
{
    ws_status s = check_common(dt, d);
    if (s != WS_OK) return s;
    if (!Kc || !Vc || !Knew || !Vnew || !pos || H < 1 || Lcap < 1 || L < 0 || m < 1) return WS_ERR_INVALID_ARG;
    if ((long long)L + m > Lcap || !(base > 0.0f) || !std::isfinite(base)) return WS_ERR_INVALID_ARG;
    if (!aligned(Kc, 16) || !aligned(Vc, 16) || !aligned(Knew, 16) || !aligned(Vnew, 16) || !aligned(pos, 4))
        return WS_ERR_INVALID_ARG;
    if ((long long)m * (d / 2) > (1 << 28)) return WS_ERR_UNSUPPORTED;
    s = check_ws(workspace, workspace_bytes, ws::inject_workspace_bytes(d, m));
    if (s != WS_OK) return s;
    const hipError_t e = ws::launch_inject(Kc, Vc, dt == WS_BF16, H, Lcap, d, L, Knew, Vnew, m, pos, base, workspace,
                                           (hipStream_t)stream);
    return e == hipSuccess ? WS_OK : WS_ERR_HIP;
}

int ws_synapse_density_is_symmetric(ws_dtype dt, int L, int d)
{
    if (check_common(dt, d) != WS_OK || L < 1) return 0;
    return ws::density_uses_symmetric(dt == WS_BF16, L, d) ? 1 : 0;
}

int ws_synapse_select_is_resident(ws_dtype dt, int H, int L, int d)
{
    ws_select_plan p;
    if (ws_synapse_select_plan(WS_SELECT_AUTO, dt, H, L, d, 0, 0, &p) != WS_OK) return 0;
    return p.resident;
}

const char *ws_status_string(ws_status s)
{
    switch (s) {
    case WS_OK: return "ok";
    case WS_ERR_INVALID_ARG: return "invalid argument";
    case WS_ERR_UNSUPPORTED: return "unsupported size or dtype";
    case WS_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case WS_ERR_HIP: return "HIP runtime or launch failure";
    case WS_ERR_TOO_LARGE: return "sizes exceed the fixed scratch of the entry point that allocates nothing";
    case WS_STATUS_INT_RANGE: break;
    }
    return "unknown status";
}

}  // extern "C"
