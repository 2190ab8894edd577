// Calls the host-only paths of the library - argument checks that return before any HIP call, and the host
// helpers - in a build whose host code is instrumented with -fsanitize=address,undefined.  No GPU is needed.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <vector>

#include "sidco.h"

static int failures = 0;
#define EXPECT(cond)                                                            \
    do {                                                                        \
        if (!(cond)) {                                                          \
            ++failures;                                                         \
            std::printf("line %d: %s\n", __LINE__, #cond);                      \
        }                                                                       \
    } while (0)

int main()
{
    alignas(16) static float buf[64];
    alignas(16) static int32_t ibuf[64];
    float* g = buf;
    float* r = buf + 16;
    int32_t* oi = ibuf;
    float* ov = buf + 32;
    int32_t* oc = ibuf + 32;
    float* oe = buf + 48;

    // argument errors are found before any HIP call
    EXPECT(sidco_compress(nullptr, nullptr, r, 16, 0.01, 0, 1, oi, ov, oc, oe) == SIDCO_ERR_NULL);
    EXPECT(sidco_compress(nullptr, g, r, 0, 0.01, 0, 1, oi, ov, oc, oe) == SIDCO_ERR_SIZE);
    EXPECT(sidco_compress(nullptr, g, r, (int64_t)1 << 31, 0.01, 0, 1, oi, ov, oc, oe) == SIDCO_ERR_SIZE);
    EXPECT(sidco_compress(nullptr, g, r, 16, 0.0, 0, 1, oi, ov, oc, oe) == SIDCO_ERR_DELTA);
    EXPECT(sidco_compress(nullptr, g, r, 16, std::nan(""), 0, 1, oi, ov, oc, oe) == SIDCO_ERR_DELTA);
    EXPECT(sidco_compress(nullptr, g, r, 16, 0.01, 7, 1, oi, ov, oc, oe) == SIDCO_ERR_DIST);
    EXPECT(sidco_compress(nullptr, g, r, 16, 0.01, 0, 0, oi, ov, oc, oe) == SIDCO_ERR_STAGES);
    EXPECT(sidco_compress(nullptr, g, r, 16, 0.01, 0, SIDCO_MAX_STAGES + 1, oi, ov, oc, oe) == SIDCO_ERR_STAGES);
    EXPECT(sidco_compress(nullptr, g, g, 16, 0.01, 0, 1, oi, ov, oc, oe) == SIDCO_ERR_ARG);
    EXPECT(sidco_compress(nullptr, (const float*)((const char*)g + 1), r, 8, 0.01, 0, 1, oi, ov, oc, oe) == SIDCO_ERR_ALIGN);
    EXPECT(sidco_compress_static(nullptr, g, r, sidco_static_max_elements() + 1, 0.01, 0, 1, oi, ov, oc, oe) == SIDCO_ERR_SIZE);
    EXPECT(sidco_compress_static(nullptr, nullptr, r, 16, 0.01, 0, 1, oi, ov, oc, oe) == SIDCO_ERR_NULL);
    const double ratios_bad[2] = {0.25, 1.5};
    const double ratios_ok[2] = {0.25, 0.04};
    EXPECT(sidco_compress_ex(nullptr, g, r, 16, 0, ratios_bad, 2, oi, ov, 16, oc, oe) == SIDCO_ERR_DELTA);
    EXPECT(sidco_compress_ex(nullptr, g, r, 16, 0, ratios_ok, 0, oi, ov, 16, oc, oe) == SIDCO_ERR_STAGES);
    EXPECT(sidco_compress_ex(nullptr, g, r, 16, 0, ratios_ok, 2, oi, ov, 0, oc, oe) == SIDCO_ERR_SIZE);
    EXPECT(sidco_compress_ex(nullptr, g, r, 16, 0, nullptr, 2, oi, ov, 16, oc, oe) == SIDCO_ERR_NULL);
    EXPECT(sidco_compress_typed(nullptr, g, 9, r, 16, 0.01, 0, 1, oi, ov, oc, oe) == SIDCO_ERR_ARG);
    EXPECT(sidco_compress_typed(nullptr, (const char*)g + 1, SIDCO_GRAD_BF16, r, 8, 0.01, 0, 1, oi, ov, oc, oe) == SIDCO_ERR_ALIGN);
    EXPECT(sidco_topk(nullptr, g, r, 16, 0, oi, ov, oc, oe) == SIDCO_ERR_SIZE);
    EXPECT(sidco_topk(nullptr, g, r, 16, 17, oi, ov, oc, oe) == SIDCO_ERR_SIZE);
    EXPECT(sidco_dgc(nullptr, g, r, 16, 0.01, 0.0, 1, oi, ov, oc, oe) == SIDCO_ERR_DELTA);
    EXPECT(sidco_scatter_add(nullptr, nullptr, 16, oi, ov, oc, 16, 1.0f) == SIDCO_ERR_NULL);
    EXPECT(sidco_scatter_add(nullptr, g, 16, oi, ov, oc, 0, 1.0f) == SIDCO_ERR_SIZE);
    EXPECT(sidco_fit(nullptr, nullptr, r, 16, 0) == SIDCO_ERR_NULL);
    EXPECT(sidco_fit_typed(nullptr, g, 5, r, 16, 0) == SIDCO_ERR_ARG);

    // batched: the plan is built (and checked) on the host before the device is touched
    const int64_t offs_bad[3] = {0, 8, 8};
    const int64_t offs_ok[3] = {0, 8, 16};
    int64_t out_offs[3] = {0, 0, 0};
    EXPECT(sidco_batched_out_offsets(offs_ok, 2, 0.5, out_offs) == SIDCO_OK);
    EXPECT(out_offs[2] == 16);
    EXPECT(sidco_batched_out_offsets(offs_ok, 0, 0.5, out_offs) == SIDCO_ERR_SIZE);
    EXPECT(sidco_batched_out_offsets(offs_ok, 2, 1.0, out_offs) == SIDCO_ERR_DELTA);
    EXPECT(sidco_compress_batched(nullptr, g, r, offs_bad, 2, 0.5, 0, 1, oi, ov, out_offs, oc, oe) == SIDCO_ERR_SIZE);
    EXPECT(sidco_compress_batched(nullptr, g, r, offs_ok, 600, 0.5, 0, 1, oi, ov, out_offs, oc, oe) == SIDCO_ERR_SIZE);
    EXPECT(sidco_compress_batched(nullptr, g, nullptr, nullptr, 2, 0.5, 0, 1, oi, ov, out_offs, oc, oe) == SIDCO_ERR_NULL);
    EXPECT(sidco_compress_batched_typed(nullptr, g, 9, r, offs_ok, 2, 0.5, 0, 1, oi, ov, out_offs, oc, oe) == SIDCO_ERR_ARG);
    EXPECT(sidco_compress_batched_typed(nullptr, (const char*)g + 1, SIDCO_GRAD_F16, r, offs_ok, 2, 0.5, 0, 1, oi, ov, out_offs, oc, oe) == SIDCO_ERR_ALIGN);
    EXPECT(sidco_workspace_bytes_batched_typed(offs_ok, 2, SIDCO_GRAD_F16, 0) > sidco_workspace_bytes_batched_typed(offs_ok, 2, SIDCO_GRAD_F16, 1));
    EXPECT(sidco_workspace_bytes_batched_typed(offs_ok, 2, 9, 0) == 0);
    EXPECT(sidco_topk_typed(nullptr, g, 9, r, 16, 4, oi, ov, oc, oe) == SIDCO_ERR_ARG);
    EXPECT(sidco_topk_typed(nullptr, (const char*)g + 2, SIDCO_GRAD_F32, r, 8, 4, oi, ov, oc, oe) == SIDCO_ERR_ALIGN);
    EXPECT(sidco_dgc_typed(nullptr, g, -1, r, 16, 0.01, 0.01, 1, oi, ov, oc, oe) == SIDCO_ERR_ARG);
    EXPECT(sidco_dgc_typed(nullptr, (const char*)g + 1, SIDCO_GRAD_BF16, r, 8, 0.01, 0.01, 1, oi, ov, oc, oe) == SIDCO_ERR_ALIGN);
    EXPECT(sidco_workspace_bytes_batched(offs_ok, 2) > 0);
    EXPECT(sidco_workspace_bytes_batched(offs_bad, 2) == 0);

    // host helpers
    double ratios[SIDCO_MAX_STAGES];
    EXPECT(sidco_stage_ratios(0.001, 3, 0.25, ratios) == 3);
    EXPECT(std::fabs(ratios[0] * ratios[1] * ratios[2] - 0.001) < 1e-15);
    EXPECT(sidco_stage_ratios(0.3, 3, 0.25, ratios) == 1 && ratios[0] == 0.3);
    EXPECT(sidco_stage_ratios(0.001, 9, 0.25, ratios) == SIDCO_ERR_STAGES);
    EXPECT(sidco_stage_ratios(0.001, 3, 0.25, nullptr) == SIDCO_ERR_NULL);
    EXPECT(sidco_out_capacity(1000, 0.01) == 1000);
    EXPECT(sidco_out_capacity(100000000, 0.001) == 4 * 100000 + 4096);
    EXPECT(sidco_out_capacity(0, 0.01) == SIDCO_ERR_SIZE);
    EXPECT(sidco_workspace_bytes(0) == 0);
    EXPECT(sidco_workspace_bytes(1000) > 16 * 1000);
    EXPECT(sidco_workspace_bytes_typed(1000, SIDCO_GRAD_BF16, 0) > sidco_workspace_bytes_typed(1000, SIDCO_GRAD_BF16, 1));
    EXPECT(sidco_workspace_bytes_typed(1000, 7, 0) == 0);
    EXPECT(sidco_adapt_stages(2, 130.0, 100.0, 0.2, 0.2, 8) == 1);
    EXPECT(sidco_adapt_stages(2, 70.0, 100.0, 0.2, 0.2, 8) == 3);
    EXPECT(sidco_adapt_stages(8, 70.0, 100.0, 0.2, 0.2, 8) == 8);
    EXPECT(sidco_adapt_stages(0, 70.0, 100.0, 0.2, 0.2, 8) == SIDCO_ERR_STAGES);
    int64_t sizes[3];
    EXPECT(sidco_dgc_sizes(1000000, 0.001, 0.01, sizes) == SIDCO_OK && sizes[0] == 10000 && sizes[1] == 10 && sizes[2] == 1000);
    EXPECT(sidco_dgc_sizes(1000000, 0.001, 0.0, sizes) == SIDCO_ERR_DELTA);
    EXPECT(sidco_set_speculation(1.5) == SIDCO_ERR_ARG);
    EXPECT(sidco_set_speculation(0.5) == SIDCO_OK);
    EXPECT(sidco_set_delta1(0.0) == SIDCO_ERR_DELTA);
    EXPECT(sidco_set_delta1(0.25) == SIDCO_OK);
    sidco_controller* c = nullptr;
    EXPECT(sidco_controller_create(&c, 0.01, 0, 1, 4, 5, 0.2, 0.2, 0.25) == SIDCO_OK && c != nullptr);
    EXPECT(sidco_controller_stages(c) == 1 && sidco_controller_iteration(c) == 0 && sidco_controller_disturbed(c) == 0);
    EXPECT(sidco_controller_compress(c, nullptr, nullptr, r, 16, oi, ov, oc, oe) == SIDCO_ERR_NULL);
    EXPECT(sidco_controller_compress_typed(c, nullptr, g, 9, r, 16, oi, ov, oc, oe) == SIDCO_ERR_ARG);
    sidco_controller_destroy(c);
    EXPECT(sidco_controller_create(&c, 0.01, 0, 5, 4, 5, 0.2, 0.2, 0.25) == SIDCO_ERR_STAGES && c == nullptr);
    EXPECT(sidco_controller_create(nullptr, 0.01, 0, 1, 4, 5, 0.2, 0.2, 0.25) == SIDCO_ERR_NULL);
    for (int code = 0; code >= -10; --code) EXPECT(sidco_strerror(code) != nullptr);
    EXPECT(sidco_version() >= 100);
    std::printf("library host paths under sanitizers: %d failures\n", failures);
    return failures ? 1 : 0;
}
