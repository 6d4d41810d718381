// Driver for the host-sanitizer build of the library's boundary (argument checks, workspace
// layout, error paths).  No GPU is needed: every call here must return before anything is
// enqueued.  The sanitizers abort on any invalid access or undefined operation in the host code.
#include <stdio.h>
#include <string.h>

#include "../../include/entmax_attn_aids.h"

#define CHECK(cond) do { if (!(cond)) { printf("failed: %s (line %d)\n", #cond, __LINE__); return 1; } } while (0)

int main() {
    CHECK(entmax_attn_mask_tile() == 64);
    CHECK(entmax_attn_histogram_bins() >= 8);
    for (int code = -8; code <= 0; ++code) CHECK(strlen(entmax_attn_strerror(code)) > 0);
    CHECK(entmax_attn_workspace_bytes(2, 16, 16384, 128, EA_BF16, 1, 0) > 0);
    CHECK(entmax_attn_workspace_bytes(2, 16, 16384, 128, EA_BF16, 1, 1) > 0);
    CHECK(entmax_attn_workspace_bytes(1, 1, 100, 64, EA_BF16, 1, 0) == 0);
    CHECK(entmax_attn_workspace_bytes(1, 1, 256, 96, EA_F32, 0, 1) == 0);
    CHECK(entmax_attn_decode_workspace_bytes(4, 8, 131072, 128, EA_BF16) > 0);
    CHECK(entmax_attn_decode_workspace_bytes(1, 1, 8, 96, EA_F32) == 0);
    CHECK(entmax_attn_decode_static_max_bytes() > 0);
    float x[4] = {0, 0, 0, 0};
    int32_t m[4] = {0, 0, 0, 0};
    alignas(256) static char ws[1024];
    // null pointers, bad alpha, bad shapes, bad dtype, short workspace: all refused before any launch
    CHECK(entmax_attn_fwd(nullptr, x, x, x, x, m, nullptr, 1, 1, 64, 64, EA_F32, 1.5f, 0, ws, sizeof ws, nullptr) == EA_ERR_NULL);
    CHECK(entmax_attn_fwd(x, x, x, x, x, m, nullptr, 1, 1, 64, 64, EA_F32, 1.0f, 0, ws, sizeof ws, nullptr) == EA_ERR_ALPHA);
    CHECK(entmax_attn_fwd(x, x, x, x, x, m, nullptr, 1, 1, 65, 64, EA_F32, 1.5f, 0, ws, sizeof ws, nullptr) == EA_ERR_SHAPE);
    CHECK(entmax_attn_fwd(x, x, x, x, x, m, nullptr, 1, 1, 64, 64, 7, 1.5f, 0, ws, sizeof ws, nullptr) == EA_ERR_DTYPE);
    CHECK(entmax_attn_fwd(x, x, x, x, x, m, nullptr, 1, 1, 64, 64, EA_F32, 1.5f, 0, ws, sizeof ws, nullptr) == EA_ERR_WORKSPACE);
    CHECK(entmax_attn_bwd(x, x, x, x, nullptr, x, m, x, x, x, 1, 1, 64, 64, EA_F32, 1.5f, 0, ws, sizeof ws, nullptr) == EA_ERR_NULL);
    CHECK(entmax_attn_bwd(x, x, x, x, x, x, m, x, x, x, 1, 1, 64, 64, EA_F32, 1.5f, 0, ws, sizeof ws, nullptr) == EA_ERR_WORKSPACE);
    const float alphas_bad[2] = {1.5f, 0.5f};
    CHECK(entmax_attn_fwd_alpha_per_head(x, x, x, x, x, m, nullptr, 1, 2, 64, 64, EA_F32, alphas_bad, 0, ws, sizeof ws, nullptr) == EA_ERR_ALPHA);
    CHECK(entmax_attn_fwd_alpha_per_head(x, x, x, x, x, m, nullptr, 1, 2, 64, 64, EA_F32, nullptr, 0, ws, sizeof ws, nullptr) == EA_ERR_NULL);
    CHECK(entmax_attn_decode(x, x, x, x, x, m, m, 1, 1, 8, 64, EA_F32, 3.5f, ws, sizeof ws, nullptr) == EA_ERR_ALPHA);
    CHECK(entmax_attn_decode(x, x, x, x, x, m, m, 1, 1, 8, 64, EA_F32, 1.5f, ws, 0, nullptr) == EA_ERR_WORKSPACE);
    CHECK(entmax_attn_decode_static(x, x, x, x, x, m, m, 1, 64, 131072, 64, EA_BF16, 1.5f, nullptr) == EA_ERR_TOO_LARGE);
    CHECK(entmax_attn_fwd_histogram_bounds(nullptr, 0, 1, 1, 64, 64, EA_F32, x, x, nullptr) == EA_ERR_NULL);
    CHECK(entmax_attn_fwd_histogram_bounds(ws, sizeof ws, 1, 1, 64, 64, EA_F32, x, x, nullptr) == EA_ERR_WORKSPACE);
    CHECK(entmax_attn_gather_enable(0) == EA_OK && entmax_attn_gather_enable(1) == EA_OK);
    float ms[EA_TIMER_SLOTS]; int launches[EA_TIMER_SLOTS];
    CHECK(entmax_attn_timer_read(ms, launches, 2) == EA_ERR_NULL);
    CHECK(entmax_attn_timer_read(ms, launches, EA_TIMER_SLOTS) == EA_OK);
    CHECK(entmax_attn_mfma_probe(nullptr, x, 4, 4, nullptr) == EA_ERR_NULL);
    printf("ok\n");
    return 0;
}
