// Driver for the sanitizer build of the library's HOST code (test infrastructure): every entry point is called with
// arguments that its validation must reject before any HIP call is made, on a machine without a GPU.  The device
// code is compiled as usual; only the host pass carries -fsanitize=address,undefined.
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "aasd.h"
#include "aasd_hooks.h"

static int g_fail = 0;
#define EXPECT(call, want)                                                                    \
    do {                                                                                      \
        const int got_ = (call);                                                              \
        if (got_ != (want)) { std::printf("%s: got %d, want %d (%s)\n", #call, got_, (int)(want), aasd_last_error()); ++g_fail; } \
    } while (0)

int main()
{
    void* P = (void*)0x10000;   // non-null, aligned, never dereferenced on the host
    int32_t* I = (int32_t*)P; uint8_t* U = (uint8_t*)P; float* F = (float*)P; uint32_t* W = (uint32_t*)P;
    EXPECT(aasd_align_sample(P, 7, 4, 100, 100, I, 2, 4, 0, 0, 0, I, U, F, F, F, I, I, U, nullptr, P, 1 << 20, nullptr), AASD_ERR_INVALID_ARG);
    EXPECT(aasd_align_sample(P, 1, 4, 100, 99, I, 2, 4, 0, 0, 0, I, U, F, F, F, I, I, U, nullptr, P, 1 << 20, nullptr), AASD_ERR_INVALID_ARG);
    EXPECT(aasd_align_sample(P, 1, 4, 100, 100, I, 2, 4, 0, 0, 0, I, U, F, F, F, I, I, U, nullptr, nullptr, 0, nullptr), AASD_ERR_WORKSPACE);
    EXPECT(aasd_align_sample(nullptr, 1, 0, 100, 100, nullptr, 2, 4, 0, 0, 0, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0, nullptr), AASD_OK);
    EXPECT(aasd_retrieve_drafts(I, 64, I, I, 2, 0, 4, 8, 4, nullptr, nullptr, 0, 0, I, I, I, I, I, nullptr, U, nullptr), AASD_ERR_INVALID_ARG);
    EXPECT(aasd_retrieve_drafts(I, 64, I, I, 2, 2, 4, 8, 4, I, nullptr, 0, 0, I, I, I, I, I, nullptr, U, nullptr), AASD_ERR_INVALID_ARG);
    EXPECT(aasd_verify(P, 1, 2, 2, 4, 100, 100, 899, I, I, nullptr, 0.1f, 0.1f, 0, I, I, I, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, P, 1 << 20, nullptr), AASD_ERR_INVALID_ARG);
    EXPECT(aasd_verify(P, 1, 2, 2, 4, 100, 100, 900, I, I, nullptr, 0.1f, 0.1f, 8, I, I, I, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, P, 1 << 20, nullptr), AASD_ERR_INVALID_ARG);
    EXPECT(aasd_verify(P, 1, 2, 2, 4, 100, 100, 900, I, I, nullptr, 0.1f, 0.1f, 2, I, I, I, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, P, 16, nullptr), AASD_ERR_WORKSPACE);
    EXPECT(aasd_verify_static(P, 1, 300, 16, 8, 100, 100, 12900, I, I, nullptr, 0.1f, 0.1f, 0, I, I, I, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr), AASD_ERR_UNSUPPORTED);
    EXPECT(aasd_verify_static(P, 1, 2, 2, 4, 100, 100, 900, I, I, nullptr, 0.1f, 0.1f, 2, I, I, I, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr), AASD_ERR_INVALID_ARG);
    EXPECT(aasd_verify_topk(P, 1, 2, 2, 4, 100, 100, 900, I, I, 9, I, I, I, nullptr, nullptr, P, 1 << 20, nullptr), AASD_ERR_INVALID_ARG);
    EXPECT(aasd_build_tree(I, I, nullptr, nullptr, 0, nullptr, 2, 4, 8, 513, I, I, I, U, I, nullptr, nullptr, nullptr), AASD_ERR_INVALID_ARG);
    EXPECT(aasd_verify_tree(P, 1, 2, 16, 100, 100, 1599, I, I, nullptr, I, 0.1f, 0.1f, 0, I, I, nullptr, I, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, P, 1 << 20, nullptr), AASD_ERR_INVALID_ARG);
    EXPECT(aasd_pool_update(P, 16, 2, 1000, 2, 4, I, 1000, I, 1, nullptr), AASD_ERR_WORKSPACE);
    EXPECT(aasd_pool_retrieve(P, 1 << 30, 2, 1000, 2, 4, I, 1000, I, I, 0, 4, nullptr, nullptr, 0, 0, I, I, I, I, I, nullptr, U, nullptr), AASD_ERR_INVALID_ARG);
    EXPECT(aasd_hook_sweep_plan(512, 1, 0), AASD_ERR_UNSUPPORTED);
    EXPECT(aasd_hook_sweep_plan(1024, 1, 4), AASD_OK);
    if (aasd_verify_workspace_bytes(1, 1, 8, 128256, 1) != 7 * 128 + 9 * 4 * 16 * 32) { std::printf("workspace query under a forced plan\n"); ++g_fail; }
    EXPECT(aasd_hook_sweep_plan(0, 0, 0), AASD_OK);
    // every size query over a grid of arguments, valid and not
    size_t total = 0;
    for (int B : {-1, 0, 1, 33, 70000})
        for (int C : {0, 1, 16, 32, 33})
            for (int k : {0, 1, 8, 16, 17})
                for (int V : {0, 1, 777, 152064})
                    total += aasd_verify_workspace_bytes(B, C, k, V, 1) + aasd_verify_topk_workspace_bytes(B, C, k, V, 0) +
                             aasd_verify_tree_workspace_bytes(B, C * 16, V, 1) + aasd_align_sample_workspace_bytes((int64_t)B * 1000, V, 1) +
                             aasd_pool_bytes(B, V, 1 + k % 8, 8);
    std::printf("%s, %d mismatches, size queries sum %zu\n", aasd_version(), g_fail, total);
    (void)W;
    return g_fail == 0 ? 0 : 1;
}
