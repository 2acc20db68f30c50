// Sanitizer driver of the HOST side of the library (CPU only, no GPU needed): everything the C ABI does
// before it touches a device -- argument validation of every entry point, the workspace layout, the
// dispatch table -- linked against a build of the library whose host code is compiled with
// -fsanitize=address,undefined (paper_2605_00837_amd/build.py: build_host_sanitized).  Exits 0 when the
// sanitizers reported nothing and every call answered as the header says.
#include <cstdio>
#include <cstring>
#include <initializer_list>

#include "../../include/fastsinkhorn.h"

static int fails = 0;
#define CHECK(cond) do { if (!(cond)) { std::fprintf(stderr, "host_sanitize_check: line %d: %s\n", __LINE__, #cond); ++fails; } } while (0)

int main() {
    CHECK(std::strlen(fs_version()) > 0);
    CHECK(fs_last_error() != nullptr);
    // workspace layout: dense and point clouds, extremes of every dimension
    const int sizes[] = {1, 2, 63, 256, 257, 1024, 1025, 4096, 8192, 16384, 16385, 65536, 1000000, FS_MAX_POINTS};
    for (int n : sizes)
        for (int m : sizes)
            for (int d : {0, 1, 3, 4, 5, 64}) {
                const size_t b = fs_workspace_bytes(n, m, d);
                CHECK(b > 0 && b % 256 == 0);
            }
    CHECK(fs_workspace_bytes(0, 5, 0) == 0 && fs_workspace_bytes(5, 5, 65) == 0 && fs_workspace_bytes(5, -1, 0) == 0);
    // dispatch table: every mode, storage type and entry-point kind over a sweep of shapes
    for (int n : sizes)
        for (int m : sizes)
            for (int d : {0, 3, 17})
                for (int km = 0; km <= 6; ++km)
                    for (int cd = 0; cd <= (d == 0 ? 2 : 0); ++cd)
                        for (int blocking = 0; blocking <= 1; ++blocking)
                            for (int cus : {1, 64, 256, 304}) {
                                fs_options o;
                                std::memset(&o, 0, sizeof(o));
                                o.kernel_mode = km;
                                o.cost_dtype = cd;
                                const int k = fs_kernel_choice(n, m, d, &o, blocking, cus);
                                CHECK((k >= FS_KERNEL_STREAM && k <= FS_KERNEL_PERSIST) || k == FS_ERR_UNSUPPORTED ||
                                      k == FS_ERR_INVALID_ARG);
                            }
    CHECK(fs_kernel_choice(8192, 8192, 0, nullptr, 1, 256) == FS_KERNEL_PERSIST);
    CHECK(fs_kernel_choice(0, 8, 0, nullptr, 1, 256) == FS_ERR_INVALID_ARG);
    CHECK(fs_kernel_choice(8, 8, 65, nullptr, 1, 256) == FS_ERR_INVALID_ARG);
    // argument validation: refused before anything is enqueued (no device is needed to get here)
    float x = 0.f;
    double y = 0.0;
    const float *p = &x;
    float *q = &x;
    CHECK(fs_sinkhorn_dense(nullptr, p, p, 4, 4, 0.1f, 10, 0.f, q, q, nullptr) == FS_ERR_INVALID_ARG);
    CHECK(fs_sinkhorn_dense(p, p, p, 0, 4, 0.1f, 10, 0.f, q, q, nullptr) == FS_ERR_INVALID_ARG);
    CHECK(fs_sinkhorn_dense(p, p, p, 4, 4, -1.f, 10, 0.f, q, q, nullptr) == FS_ERR_INVALID_ARG);
    CHECK(fs_sinkhorn_dense(p, p, p, 4, 4, 0.1f, -1, 0.f, q, q, nullptr) == FS_ERR_INVALID_ARG);
    CHECK(fs_sinkhorn_dense(p, nullptr, p, 4, 4, 0.1f, 10, 0.f, q, q, nullptr) == FS_ERR_INVALID_ARG);
    CHECK(fs_sinkhorn_dense(p, p, p, 4, 4, 0.1f, 10, 0.f, nullptr, q, nullptr) == FS_ERR_INVALID_ARG);
    CHECK(fs_sinkhorn_points(p, nullptr, 3, p, p, 4, 4, 0.1f, 10, 0.f, q, q, nullptr) == FS_ERR_INVALID_ARG);
    CHECK(fs_sinkhorn_points(p, p, 0, p, p, 4, 4, 0.1f, 10, 0.f, q, q, nullptr) == FS_ERR_INVALID_ARG);
    CHECK(fs_sinkhorn_points(p, p, 65, p, p, 4, 4, 0.1f, 10, 0.f, q, q, nullptr) == FS_ERR_INVALID_ARG);
    CHECK(fs_sinkhorn_solve(p, p, p, 3, p, p, 4, 4, 0.1f, 10, 0.f, q, q, nullptr, nullptr, nullptr) == FS_ERR_INVALID_ARG);
    CHECK(fs_sinkhorn_dense_ex(p, p, p, 4, FS_MAX_POINTS + 1, 0.1f, 10, 0.f, q, q, nullptr, nullptr, q, 1 << 20, nullptr) ==
          FS_ERR_INVALID_ARG);
    CHECK(fs_sinkhorn_dense_ex(p, p, p, 300, 300, 0.1f, 10, 0.f, q, q, nullptr, nullptr, nullptr, 0, nullptr) == FS_ERR_WORKSPACE);
    CHECK(fs_sinkhorn_dense_static(p, p, p, 12288, 12288, 0.1f, 10, 0.f, q, q, nullptr, nullptr, nullptr) == FS_ERR_WORKSPACE);
    CHECK(std::strstr(fs_last_error(), "static buffer") != nullptr);
    CHECK(fs_sinkhorn_dense_static(nullptr, p, p, 8, 8, 0.1f, 10, 0.f, q, q, nullptr, nullptr, nullptr) == FS_ERR_INVALID_ARG);
    {
        fs_options o;
        std::memset(&o, 0, sizeof(o));
        o.cost_dtype = 3;
        CHECK(fs_sinkhorn_solve(p, nullptr, nullptr, 0, p, p, 8, 8, 0.1f, 10, 0.f, q, q, nullptr, &o, nullptr) == FS_ERR_INVALID_ARG);
        o.cost_dtype = 1;
        CHECK(fs_sinkhorn_solve(p, nullptr, nullptr, 0, p, p, 8, 12, 0.1f, 10, 0.f, q, q, nullptr, &o, nullptr) == FS_ERR_UNSUPPORTED);
        o.cost_dtype = 0;
        o.kernel_mode = 9;
        CHECK(fs_sinkhorn_solve(p, nullptr, nullptr, 0, p, p, 8, 8, 0.1f, 10, 0.f, q, q, nullptr, &o, nullptr) == FS_ERR_INVALID_ARG);
    }
    CHECK(fs_sinkhorn_dense_batched(p, p, p, 0, 8, 8, 0.1f, 10, 0.f, q, q, nullptr, nullptr, nullptr) == FS_ERR_INVALID_ARG);
    CHECK(fs_sinkhorn_dense_batched(p, p, p, 2, 300, 8, 0.1f, 10, 0.f, q, q, nullptr, nullptr, nullptr) == FS_ERR_UNSUPPORTED);
    CHECK(fs_sinkhorn_annealed(p, nullptr, nullptr, 0, p, p, 8, 8, 0.1f, 0.05f, 0.5f, 5, 10, 0.f, q, q, nullptr, nullptr,
                               nullptr, nullptr) == FS_ERR_INVALID_ARG);
    CHECK(fs_plan(p, nullptr, nullptr, 0, p, p, 8, 8, 0.1f, p, p, nullptr, nullptr) == FS_ERR_INVALID_ARG);
    CHECK(fs_cost(p, nullptr, nullptr, 0, p, p, 8, 8, 0.1f, nullptr, p, &y, nullptr) == FS_ERR_INVALID_ARG);
    CHECK(fs_plan_f64(p, nullptr, nullptr, 0, p, p, 8, 8, 0.1f, nullptr, &y, q, nullptr) == FS_ERR_INVALID_ARG);
    CHECK(fs_cost_f64(p, nullptr, nullptr, 0, p, p, 8, 8, 0.1f, &y, &y, nullptr, nullptr) == FS_ERR_INVALID_ARG);
    CHECK(fs_diagnostics(p, nullptr, nullptr, 0, p, p, 8, 8, 0.1f, p, nullptr, nullptr, nullptr, &y, nullptr, nullptr, nullptr) ==
          FS_ERR_INVALID_ARG);
    CHECK(fs_barycentric(p, nullptr, nullptr, 0, p, p, 8, 8, 0.1f, p, p, nullptr, nullptr, p, 9, q, nullptr) == FS_ERR_INVALID_ARG);
    CHECK(fs_update_f(p, nullptr, nullptr, 0, p, p, 8, 8, 0.1f, nullptr, &y, nullptr) == FS_ERR_INVALID_ARG);
    CHECK(fs_update_g(p, nullptr, nullptr, 0, p, p, 8, 8, 0.1f, &y, nullptr, nullptr) == FS_ERR_INVALID_ARG);
    CHECK(fs_last_kernel_timing(nullptr, nullptr, nullptr, nullptr) == FS_ERR_INVALID_ARG);
    {
        float us = 0.0f;
        CHECK(fs_read_rate(nullptr, 1 << 20, 3, &us, nullptr) == FS_ERR_INVALID_ARG);
        CHECK(fs_read_rate(p, 1 << 20, 0, &us, nullptr) == FS_ERR_INVALID_ARG);
        CHECK(fs_read_rate(p, 8, 3, &us, nullptr) == FS_ERR_INVALID_ARG);
        CHECK(fs_read_rate(p, 1 << 20, 3, nullptr, nullptr) == FS_ERR_INVALID_ARG);
    }
    fs_clear_cache();
    if (fails) { std::fprintf(stderr, "host_sanitize_check: %d check(s) failed\n", fails); return 1; }
    std::printf("host_sanitize_check: ok\n");
    return 0;
}
