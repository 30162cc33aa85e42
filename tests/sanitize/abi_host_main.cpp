// Driver for a host-only sanitizer build of libobc (its host code compiled with
// -fsanitize=address,undefined and no device code at all): every entry point that does no GPU work
// -- the workspace queries, the version / error strings and the argument checks that reject a call
// before anything is launched -- is called with valid and invalid arguments.  Exit status 0 = clean.
#include <cstdio>
#include <cstring>
#include <initializer_list>

#include "obc.h"

#define EXPECT(cond) do { if (!(cond)) { std::fprintf(stderr, "failed: %s\n", #cond); return 1; } } while (0)

int main()
{
    size_t n = 0;
    EXPECT(std::strstr(obc_version(), "gfx950") != nullptr);
    EXPECT(std::strcmp(obc_last_error(nullptr), "null context") == 0);
    const int widths[] = {1, 32, 192, 193, 576, 768, 2304, 3072, 4608, 5000};
    for (int d : widths)
        for (int R : {0, 1, 64, 3072})
            for (int strategy : {OBC_STRATEGY_AUTO, OBC_STRATEGY_RANK1, OBC_STRATEGY_BLOCKED}) {
                int rc = obc_rows_workspace_bytes(R, d, strategy, &n);
                EXPECT(rc == OBC_OK || rc == OBC_ERR_BAD_SHAPE);
                for (int c : {1, 2, 4, 8}) {
                    rc = obc_blocks_workspace_bytes(R, d, c, strategy, &n);
                    EXPECT(rc == OBC_OK || rc == OBC_ERR_BAD_SHAPE || rc == OBC_ERR_BAD_ARG);
                }
            }
    EXPECT(obc_rows_workspace_bytes(-1, 32, 0, &n) == OBC_ERR_BAD_ARG);
    EXPECT(obc_rows_workspace_bytes(1, 32, 0, nullptr) == OBC_ERR_BAD_ARG);
    EXPECT(obc_rows_workspace_bytes(1, 32, 9, &n) == OBC_ERR_BAD_ARG);
    EXPECT(obc_blocks_workspace_bytes(8, 576, 9, 0, &n) == OBC_ERR_BAD_ARG);
    EXPECT(obc_invert_workspace_bytes(0, &n) == OBC_ERR_BAD_ARG);
    EXPECT(obc_invert_workspace_bytes(4608, &n) == OBC_OK && n >= (size_t)2 * 4608 * 4608 * 8);
    EXPECT(obc_hessian_workspace_bytes(4608, 100000, &n) == OBC_OK && n >= (size_t)4608 * 4608 * 4);
    EXPECT(obc_hessian_workspace_bytes(0, 10, &n) == OBC_ERR_BAD_ARG);
    EXPECT(obc_cross_workspace_bytes(256, 2304, 50000, &n) == OBC_OK);
    EXPECT(obc_cross_workspace_bytes(0, 2304, 50000, &n) == OBC_ERR_BAD_ARG);
    EXPECT(obc_refit_workspace_bytes(576, 64, &n) == OBC_OK);
    EXPECT(obc_refit_workspace_bytes(576, 0, &n) == OBC_ERR_BAD_ARG);
    EXPECT(obc_global_select_workspace_bytes(3072, 768, &n) == OBC_OK && n <= (size_t)OBC_SELECT_STATIC_SCRATCH_BYTES);
    EXPECT(obc_global_select_workspace_bytes(OBC_SELECT_STATIC_MAX_ROWS, OBC_SELECT_STATIC_MAX_WEIGHTS / OBC_SELECT_STATIC_MAX_ROWS, &n) == OBC_OK &&
           n <= (size_t)OBC_SELECT_STATIC_SCRATCH_BYTES);
    EXPECT(obc_global_select_workspace_bytes(4, 0, &n) == OBC_ERR_BAD_ARG);
    EXPECT(obc_reconstruct_workspace_bytes(256, 2304, 1152, &n) == OBC_OK && n >= (size_t)256 * 1152 * 1152 * 8);
    EXPECT(obc_reconstruct_workspace_bytes(4, 32, 0, &n) == OBC_OK);
    EXPECT(obc_reconstruct_workspace_bytes(4, 32, 33, &n) == OBC_ERR_BAD_ARG);
    // a null context is refused before anything else is looked at
    float f = 0.f;
    int32_t i32 = 0;
    uint8_t u8 = 0;
    double ms = 0.0;
    EXPECT(obc_destroy(nullptr) == OBC_ERR_BAD_ARG);
    EXPECT(obc_check(nullptr) == OBC_ERR_BAD_ARG);
    EXPECT(obc_create(nullptr, nullptr) == OBC_ERR_BAD_ARG);
    EXPECT(obc_profile_begin(nullptr) == OBC_ERR_BAD_ARG);
    EXPECT(obc_profile_end(nullptr, nullptr) == OBC_ERR_BAD_ARG);
    EXPECT(obc_membench(nullptr, 0, 0, &f, &f, 16, 1, &ms) == OBC_ERR_BAD_ARG);
    EXPECT(obc_mfmabench(nullptr, 0, 1, 1, &ms, &ms) == OBC_ERR_BAD_ARG);
    EXPECT(obc_hessian(nullptr, &f, 1, 1, 1, 0.f, 0, &f, &f, 4) == OBC_ERR_BAD_ARG);
    EXPECT(obc_invert(nullptr, &f, 1, &f, 4) == OBC_ERR_BAD_ARG);
    EXPECT(obc_cross(nullptr, &f, &f, 1, 1, 1, 1, 1, 0, &f, &f, 4) == OBC_ERR_BAD_ARG);
    EXPECT(obc_refit(nullptr, &f, 1, &f, 1, &f, 0, &f, 4) == OBC_ERR_BAD_ARG);
    EXPECT(obc_prune_rows(nullptr, &f, &f, 1, 1, 1, 0, 0, nullptr, nullptr, &i32, &f, &f, nullptr, 0, &f, 4) == OBC_ERR_BAD_ARG);
    EXPECT(obc_prune_blocks(nullptr, &f, &f, 1, 4, 4, 1, nullptr, &i32, &f, &f, nullptr, 0, &f, 4) == OBC_ERR_BAD_ARG);
    EXPECT(obc_quant_rows(nullptr, &f, &f, 1, 1, &f, &f, 15, nullptr, 0, &i32, &f, &i32, &f, 0, &f, 4) == OBC_ERR_BAD_ARG);
    EXPECT(obc_minmax_grid(nullptr, &f, nullptr, 1, 1, 15, 0, &f, &f) == OBC_ERR_BAD_ARG);
    EXPECT(obc_global_select(nullptr, &f, &i32, 1, 1, 0, &i32, &u8, &f, 4) == OBC_ERR_BAD_ARG);
    EXPECT(obc_global_select_static(nullptr, &f, &i32, 1, 1, 0, &i32, &u8) == OBC_ERR_BAD_ARG);
    EXPECT(obc_gather_trace(nullptr, &f, &f, &i32, 1, 1, 1, &f) == OBC_ERR_BAD_ARG);
    EXPECT(obc_reconstruct_rows(nullptr, &f, &f, &u8, 1, 1, 1, &f, &f, 4) == OBC_ERR_BAD_ARG);
    std::puts("libobc host sanitizer run clean");
    return 0;
}
