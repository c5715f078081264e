// Exercises the GPU-free part of the C ABI (layout tables, colour trees, roles, schedule,
// options, error strings) so that it can be run under AddressSanitizer / UBSan on the host.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "mc.h"
#include "mc_tiles.h"

#define REQUIRE(c)                                                    \
    do {                                                              \
        if (!(c)) {                                                   \
            std::printf("host_driver: failed %s (line %d)\n", #c, __LINE__); \
            return 1;                                                 \
        }                                                             \
    } while (0)

int main() {
    for (int32_t k : {1, 2, 3, 7, 64, 1000}) {
        for (int32_t n : {1, 2, 5, 161, 700}) {
            std::vector<int64_t> numel(n);
            for (int32_t t = 0; t < n; ++t) numel[t] = (int64_t(t) * 2654435761u) % 70001;
            if (n > 2) numel[1] = 0;
            mc_layout* L = nullptr;
            REQUIRE(mc_layout_create(numel.data(), n, k, &L) == MC_OK && L);
            int64_t N = -1;
            int32_t nn = 0, kk = 0;
            REQUIRE(mc_layout_total(L, &N) == MC_OK);
            REQUIRE(mc_layout_counts(L, &nn, &kk) == MC_OK && nn == n && kk == k);
            std::vector<int64_t> off(n + 1), b(k + 1);
            REQUIRE(mc_layout_tensor_offsets(L, off.data()) == MC_OK);
            REQUIRE(mc_layout_colour_bounds(L, b.data()) == MC_OK);
            REQUIRE(off[0] == 0 && off[n] == N && b[0] == 0 && b[k] == N);
            for (int32_t c = 0; c < k; ++c) REQUIRE(b[c] <= b[c + 1]);
            // argument validation paths that return before any GPU call
            std::vector<const void*> ptrs(n, reinterpret_cast<const void*>(0x10000000));
            REQUIRE(mc_pack(L, ptrs.data(), reinterpret_cast<void*>(0x10000004), nullptr) != MC_OK || N == 0);
            std::vector<int32_t> order(size_t(k) * 3, 0);
            const void* x[3] = {ptrs[0], ptrs[0], ptrs[0]};
            REQUIRE(mc_reduce_update(L, x, 3, order.data(), nullptr, nullptr, nullptr, 0.1f, 0.9f, 0.f, nullptr) ==
                    MC_ERR_INVALID_ARG);
            REQUIRE(mc_layout_destroy(L) == MC_OK);
        }
    }
    mc_layout* bad = reinterpret_cast<mc_layout*>(1);
    int64_t neg[2] = {4, -1};
    REQUIRE(mc_layout_create(neg, 2, 1, &bad) == MC_ERR_INVALID_ARG && bad == nullptr);
    REQUIRE(mc_layout_destroy(nullptr) == MC_OK);

    for (int32_t n = 1; n < 80; ++n) {
        for (int32_t k = 1; k < 12; ++k) {
            std::vector<int32_t> parent(size_t(n) * k, -7), role(k), cnt(k), ch(size_t(k) * k);
            const int rc = mc_colour_trees(n, k, parent.data());
            if (rc != MC_OK) {
                REQUIRE(mc_rank_roles(n, k, 0, role.data(), cnt.data(), ch.data()) == MC_ERR_INVALID_ARG);
                continue;
            }
            for (int32_t c = 0; c < k; ++c) {
                int roots = 0;
                for (int32_t r = 0; r < n; ++r) {
                    const int32_t p = parent[size_t(c) * n + r];
                    REQUIRE(p >= -1 && p < n);
                    roots += p == -1;
                }
                REQUIRE(roots == 1);
            }
            for (int32_t r = 0; r < n; ++r) REQUIRE(mc_rank_roles(n, k, r, role.data(), cnt.data(), ch.data()) == MC_OK);
        }
    }
    // The die-aware tile order is a permutation of the launch's tiles for every grid and run length,
    // and inside a full span die x (workgroups x, x+8, ...) walks consecutive tiles.
    for (int n : {0, 1, 7, 8, 63, 64, 65, 1000, 6834, 12479}) {
        for (int run : {0, 1, 2, 3, 8, 16, 64}) {
            std::vector<char> seen(size_t(n), 0);
            for (int b = 0; b < n; ++b) {
                const int t = mc::xcd_tile(b, n, run);
                REQUIRE(t >= 0 && t < n && !seen[t]);
                seen[t] = 1;
                if (run > 1 && b + mc::kXcds < n - n % (mc::kXcds * run) && (b % (mc::kXcds * run)) / mc::kXcds < run - 1)
                    REQUIRE(mc::xcd_tile(b + mc::kXcds, n, run) == t + 1);
            }
        }
    }
    float lr = 0.f;
    REQUIRE(mc_lr_schedule(0.1f, 32, 256, 5.f, 30.f, 31.f, &lr) == MC_OK && lr > 0.31f && lr < 0.33f);
    REQUIRE(mc_lr_schedule(0.1f, 0, 256, 5.f, 30.f, 31.f, &lr) == MC_ERR_INVALID_ARG);
    int v = 0;
    REQUIRE(mc_get_option(MC_OPT_RU_SHAPE, &v) == MC_OK && mc_set_option(MC_OPT_RU_SHAPE, v) == MC_OK);
    REQUIRE(mc_set_option(12345, 1) == MC_ERR_INVALID_ARG);
    for (int code = -7; code <= 1; ++code) REQUIRE(mc_strerror(code) != nullptr);
    std::printf("host_driver: ok\n");
    return 0;
}
