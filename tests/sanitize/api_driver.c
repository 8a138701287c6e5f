/* Calls every entry point of include/ws_synapse.h with bad and with well-formed arguments against stub
 * launchers (api_stubs.cpp), inside a build with -fsanitize=address,undefined: the front end must reject what
 * it documents, reach the launcher otherwise, and do neither out-of-bounds reads of the host arrays it is
 * given (sigma) nor undefined arithmetic on the sizes. */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

#include "../../include/ws_synapse.h"

extern int g_launches;
static int failures = 0;
#define CHECK(cond) do { if (!(cond)) { printf("FAILED line %d: %s\n", __LINE__, #cond); ++failures; } } while (0)

int main(void)
{
    void *fake = (void *)0x10000, *odd = (void *)0x10004;
    const size_t big = (size_t)1 << 40;
    const int H = 3;
    float *sigma = malloc(sizeof(float) * H);      /* heap: a read past H is an ASan report */
    for (int h = 0; h < H; ++h) sigma[h] = 1.5f;

    CHECK(ws_synapse_density(fake, WS_BF16, H, 1000, 64, sigma, fake, fake, big, NULL) == WS_OK);
    CHECK(ws_synapse_density(fake, WS_BF16, H, 1000, 64, sigma, fake, fake, 100, NULL) == WS_ERR_WORKSPACE);
    CHECK(ws_synapse_density(fake, WS_BF16, H, 1000, 64, sigma, fake, odd, big, NULL) == WS_ERR_WORKSPACE);
    CHECK(ws_synapse_density(NULL, WS_BF16, H, 1000, 64, sigma, fake, fake, big, NULL) == WS_ERR_INVALID_ARG);
    CHECK(ws_synapse_density(fake, WS_BF16, H, 1000, 100, sigma, fake, fake, big, NULL) == WS_ERR_UNSUPPORTED);
    CHECK(ws_synapse_density(fake, WS_BF16, H, 1 << 24, 64, sigma, fake, fake, big, NULL) == WS_ERR_UNSUPPORTED);
    CHECK(ws_synapse_density(fake, WS_BF16, H, 2147483647, 64, sigma, fake, fake, big, NULL) == WS_ERR_UNSUPPORTED);
    CHECK(ws_synapse_density(fake, WS_BF16, -2147483647 - 1, 1000, 64, sigma, fake, fake, big, NULL) == WS_ERR_INVALID_ARG);
    sigma[2] = 0.0f;
    CHECK(ws_synapse_density(fake, WS_BF16, H, 1000, 64, sigma, fake, fake, big, NULL) == WS_ERR_INVALID_ARG);
    sigma[2] = NAN;
    CHECK(ws_synapse_density(fake, WS_F32, H, 1000, 128, sigma, fake, fake, big, NULL) == WS_ERR_INVALID_ARG);
    sigma[2] = 1e-30f;     /* 1/sigma^2 overflows the exponent scale */
    CHECK(ws_synapse_density(fake, WS_F32, H, 1000, 128, sigma, fake, fake, big, NULL) == WS_ERR_INVALID_ARG);
    sigma[2] = 2.0f;
    int flagged = -1;
    CHECK(ws_synapse_density_check(NULL, H, NULL, &flagged, NULL) == WS_ERR_INVALID_ARG);
    CHECK(ws_synapse_density_check(fake, 0, NULL, &flagged, NULL) == WS_ERR_INVALID_ARG);
    CHECK(ws_synapse_density_check(fake, H, NULL, NULL, NULL) == WS_ERR_INVALID_ARG);
    CHECK(ws_synapse_density_is_symmetric(WS_BF16, 32768, 64) == 1 && ws_synapse_density_is_symmetric(WS_F32, 32768, 64) == 0);
    CHECK(ws_synapse_density_is_symmetric(WS_BF16, 32768, 72) == 0);
    const int before = g_launches;

    CHECK(ws_synapse_select(fake, WS_BF16, H, 1000, 64, fake, 20, 0.5f, fake, NULL, fake, big, NULL) == WS_OK);
    CHECK(ws_synapse_select(fake, WS_BF16, H, 1000, 64, fake, 1001, 0.5f, fake, NULL, fake, big, NULL) == WS_ERR_INVALID_ARG);
    CHECK(ws_synapse_select(fake, WS_BF16, H, 1000, 64, fake, 20, -0.1f, fake, NULL, fake, big, NULL) == WS_ERR_INVALID_ARG);
    CHECK(ws_synapse_select(fake, WS_BF16, H, 1000, 64, fake, 20, NAN, fake, NULL, fake, big, NULL) == WS_ERR_INVALID_ARG);
    CHECK(ws_synapse_select(fake, WS_BF16, H, 1000, 64, fake, 20, 0.5f, fake, NULL, NULL, 0, NULL) == WS_ERR_WORKSPACE);
    CHECK(ws_synapse_select_with(WS_SELECT_RESIDENT, fake, WS_F32, H, 1000, 64, fake, 20, 0.5f, fake, fake, fake, big, NULL) ==
          WS_ERR_UNSUPPORTED);
    CHECK(ws_synapse_select_with(WS_SELECT_STREAMING, fake, WS_F32, H, 1000, 64, fake, 20, 1.0f, fake, fake, fake, big, NULL) ==
          WS_OK);
    CHECK(ws_synapse_select_with((ws_select_kernel)5, fake, WS_F32, H, 1000, 64, fake, 20, 1.0f, fake, fake, fake, big, NULL) ==
          WS_ERR_INVALID_ARG);
    ws_select_plan plan;
    CHECK(ws_synapse_select_plan(WS_SELECT_AUTO, WS_BF16, H, 1000, 64, 64, 2, &plan) == WS_OK && plan.compute_units == 64);
    CHECK(ws_synapse_select_plan(WS_SELECT_AUTO, WS_BF16, H, 1000, 64, 64, 2, NULL) == WS_ERR_INVALID_ARG);
    CHECK(ws_synapse_select_plan(WS_SELECT_RESIDENT, WS_BF16, H, 100000, 64, 0, 0, &plan) == WS_ERR_UNSUPPORTED);
    int failed = -1;
    CHECK(ws_synapse_select_failed(NULL, NULL, &failed) == WS_ERR_HIP);      /* no device here: no static scratch */
    CHECK(ws_synapse_select_static(fake, WS_BF16, H, 1000, 64, fake, 1001, 0.5f, fake, NULL, NULL) == WS_ERR_INVALID_ARG);
    CHECK(ws_synapse_select_static(fake, WS_F32, H, 2000000, 64, fake, 20, 0.5f, fake, NULL, NULL) == WS_ERR_TOO_LARGE);
    CHECK(ws_synapse_select_static(fake, WS_BF16, H, 1000, 64, fake, 20, 0.5f, fake, NULL, NULL) == WS_ERR_HIP);
    CHECK(ws_synapse_select_failed(fake, NULL, NULL) == WS_ERR_INVALID_ARG);

    CHECK(ws_synapse_gather(fake, fake, WS_BF16, H, 1000, 64, fake, 20, fake, fake, NULL) == WS_OK);
    CHECK(ws_synapse_gather(fake, fake, WS_BF16, H, 1000, 64, fake, 0, fake, fake, NULL) == WS_ERR_INVALID_ARG);
    CHECK(ws_synapse_gather(fake, odd, WS_BF16, H, 1000, 64, fake, 20, fake, fake, NULL) == WS_ERR_INVALID_ARG);

    CHECK(ws_synapse_attend(fake, fake, fake, WS_BF16, 100, 12, 3, 20, 64, 0.0f, fake, NULL, 0, NULL) == WS_OK);
    CHECK(ws_synapse_attend(fake, fake, fake, WS_BF16, 100, 12, 5, 20, 64, 0.0f, fake, NULL, 0, NULL) == WS_ERR_INVALID_ARG);
    CHECK(ws_synapse_attend(fake, fake, fake, WS_BF16, 100, 12, 3, 20, 64, INFINITY, fake, NULL, 0, NULL) == WS_ERR_INVALID_ARG);
    CHECK(ws_synapse_attend(fake, fake, fake, WS_BF16, 100, 70000, 70000, 20, 64, 0.0f, fake, NULL, 0, NULL) == WS_ERR_UNSUPPORTED);
    CHECK(ws_synapse_attend(fake, fake, fake, WS_BF16, 256, 32, 8, 2621, 128, 0.0f, fake, NULL, 0, NULL) == WS_ERR_WORKSPACE);
    CHECK(ws_synapse_attend(fake, fake, fake, WS_BF16, 256, 32, 8, 2621, 128, 0.0f, fake, fake, big, NULL) == WS_OK);
    CHECK(ws_synapse_attend_indexed(fake, fake, fake, fake, WS_BF16, 100, 12, 3, 4096, 20, 64, 0.0f, fake, NULL, 0, NULL) == WS_OK);
    CHECK(ws_synapse_attend_indexed(fake, fake, fake, NULL, WS_BF16, 100, 12, 3, 4096, 20, 64, 0.0f, fake, NULL, 0, NULL) == WS_ERR_INVALID_ARG);
    CHECK(ws_synapse_attend_indexed(fake, fake, fake, fake, WS_BF16, 100, 12, 3, 0, 20, 64, 0.0f, fake, NULL, 0, NULL) == WS_ERR_INVALID_ARG);
    CHECK(ws_synapse_attend_indexed(fake, fake, fake, fake, WS_F32, 100, 12, 3, 1 << 23, 20, 128, 0.0f, fake, NULL, 0, NULL) == WS_ERR_UNSUPPORTED);
    CHECK(ws_synapse_attend_indexed(fake, fake, fake, fake, WS_BF16, 256, 32, 8, 131072, 2621, 128, 0.0f, fake, NULL, 0, NULL) == WS_ERR_WORKSPACE);

    CHECK(ws_synapse_attention_mass(fake, fake, WS_BF16, 2, 4, 8, 1000, 64, 0.0f, 1, fake, fake, big, NULL) == WS_OK);
    CHECK(ws_synapse_attention_mass(fake, fake, WS_BF16, 2, 4, 6, 1000, 64, 0.0f, 1, fake, fake, big, NULL) == WS_ERR_INVALID_ARG);
    CHECK(ws_synapse_attention_mass(fake, fake, WS_BF16, 70000, 4, 8, 1000, 64, 0.0f, 1, fake, fake, big, NULL) ==
          WS_ERR_UNSUPPORTED);
    CHECK(ws_synapse_attention_mass(fake, fake, WS_BF16, 2, 4, 8, 1000, 64, 0.0f, 1, fake, fake, 16, NULL) == WS_ERR_WORKSPACE);

    CHECK(ws_synapse_density_append(fake, WS_BF16, H, 1000, 64, 4, sigma, fake, fake, fake, big, NULL) == WS_OK);
    CHECK(ws_synapse_density_append(fake, WS_BF16, H, 1000, 64, 33, sigma, fake, fake, fake, big, NULL) == WS_ERR_UNSUPPORTED);
    CHECK(ws_synapse_density_append(fake, WS_BF16, H, 1000, 64, 1000, sigma, fake, fake, fake, big, NULL) == WS_ERR_INVALID_ARG);

    CHECK(ws_synapse_gate(fake, fake, WS_BF16, 100, 896, 0.5f, fake, fake, NULL) == WS_OK);
    CHECK(ws_synapse_gate(fake, fake, WS_BF16, 100, 896, NAN, fake, fake, NULL) == WS_ERR_INVALID_ARG);
    CHECK(ws_synapse_gate(fake, fake, WS_BF16, 2147483647, 896, 0.5f, fake, fake, NULL) == WS_OK);

    CHECK(ws_synapse_inject(fake, fake, WS_BF16, H, 1000, 64, 990, fake, fake, 10, fake, 1e6f, fake, big, NULL) == WS_OK);
    CHECK(ws_synapse_inject(fake, fake, WS_BF16, H, 1000, 64, 995, fake, fake, 10, fake, 1e6f, fake, big, NULL) ==
          WS_ERR_INVALID_ARG);
    CHECK(ws_synapse_inject(fake, fake, WS_BF16, H, 2147483647, 64, 2147483647, fake, fake, 10, fake, 1e6f, fake, big, NULL) ==
          WS_ERR_INVALID_ARG);   /* L + m must not wrap */
    CHECK(ws_synapse_inject(fake, fake, WS_BF16, H, 1000, 64, 0, fake, fake, 10, fake, -1.0f, fake, big, NULL) ==
          WS_ERR_INVALID_ARG);

    for (int op = 0; op <= 7; ++op) {
        (void)ws_synapse_workspace_bytes((ws_op)op, WS_BF16, H, 1000, 64, 20, 100, 12);
        (void)ws_synapse_workspace_bytes((ws_op)op, WS_BF16, 2147483647, 16777215, 128, 2147483647, 2147483647, 2147483647);
        CHECK(ws_synapse_workspace_bytes((ws_op)op, WS_BF16, H, 1000, 96, 20, 100, 12) == (size_t)-1);
    }
    CHECK(ws_synapse_workspace_bytes(WS_OP_DENSITY, WS_BF16, 0, 1000, 64, 1, 1, 1) == (size_t)-1);
    for (int s = 0; s <= 8; ++s) CHECK(ws_status_string((ws_status)s) != NULL);
    CHECK(ws_synapse_select_is_resident(WS_BF16, H, 1000, 64) == 1);
    CHECK(g_launches - before == 11);

    free(sigma);
    printf(failures ? "%d check(s) failed\n" : "all checks passed\n", failures);
    return failures ? 1 : 0;
}
