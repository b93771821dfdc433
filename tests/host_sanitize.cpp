// CPU-only driver for tests/test_host_sanitizer.py: the host side of libpamm (sampler, launch planners, workspace
// arithmetic, every argument check) compiled with -fsanitize=address,undefined and run over ordinary, extreme and
// invalid arguments.  Prints "clean" when it reaches the end; a sanitizer report aborts it before that.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../paper_2506_02939_amd/csrc/api.cpp"

#define REQUIRE(cond)                                                          \
    do {                                                                       \
        if (!(cond)) {                                                         \
            std::fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, #cond);    \
            std::exit(1);                                                      \
        }                                                                      \
    } while (0)

int main() {
    // ---- sampler: small, k = b, the largest b, the largest k
    {
        std::vector<int32_t> idx(16384);
        const int64_t bs[] = {1, 2, 7, 64, 4096, 16384, 65536, (int64_t(1) << 31) - 1};
        for (int64_t b : bs)
            for (int64_t k : {int64_t(1), int64_t(2), int64_t(63), int64_t(1024), int64_t(16384)}) {
                if (k > b) continue;
                for (uint64_t seed : {uint64_t(0), uint64_t(12345), ~uint64_t(0)}) {
                    REQUIRE(pamm_sample_indices(b, k, seed, idx.data()) == PAMM_OK);
                    for (int64_t j = 0; j < k; ++j) REQUIRE(idx[j] >= 0 && idx[j] < b);
                }
            }
        std::vector<char> seen(4096, 0);
        REQUIRE(pamm_sample_indices(4096, 4096, 3, idx.data()) == PAMM_OK);
        for (int j = 0; j < 4096; ++j) { REQUIRE(!seen[idx[j]]); seen[idx[j]] = 1; }
        REQUIRE(pamm_sample_indices(4, 5, 0, idx.data()) == PAMM_ERR_INVALID_ARG);
        REQUIRE(pamm_sample_indices(int64_t(1) << 31, 5, 0, idx.data()) == PAMM_ERR_INVALID_ARG);
        REQUIRE(pamm_sample_indices(4, 2, 0, nullptr) == PAMM_ERR_INVALID_ARG);
        std::vector<uint64_t> draws(1000);
        for (uint64_t range : {uint64_t(1), uint64_t(5), uint64_t(3) << 62, (uint64_t(1) << 63) + 12345, ~uint64_t(0)}) {
            REQUIRE(pamm_debug_bounded(7, range, 1000, draws.data()) == PAMM_OK);
            for (uint64_t v : draws) REQUIRE(v < range);
        }
        REQUIRE(pamm_debug_bounded(7, 0, 1, draws.data()) == PAMM_ERR_INVALID_ARG);
        REQUIRE(pamm_debug_bounded(7, 5, 1, nullptr) == PAMM_ERR_INVALID_ARG);
    }

    // ---- planners and workspace queries over ordinary and extreme sizes, with and without overrides
    const int64_t big = (int64_t(1) << 31) - 8;
    const pamm_debug_plan plans[] = {{0, 0, 0, 0, 0, 0}, {1, 2, 16, 1, 1, 0}, {8, 8, 4096, 3, 16384, 1}, {3, 5, 17, 9, -4, 0}, {0, 0, 0, 0, 0, 1}};
    for (const pamm_debug_plan& pp : plans) {
        REQUIRE(pamm_debug_set_plan(&pp) == PAMM_OK);
        for (pamm_dtype dt : {PAMM_F32, PAMM_BF16})
            for (int64_t b : {int64_t(1), int64_t(100), int64_t(8192), int64_t(65536), int64_t(1500003), big})
                for (int64_t k : {int64_t(1), int64_t(16), int64_t(300), int64_t(2100), int64_t(16384)}) {
                    if (k > b) continue;
                    for (int64_t n : {int64_t(8), int64_t(2048), big}) {
                        pamm::CompressPlan cp;
                        REQUIRE(pamm::plan_compress(b, n, k, dt, &cp) == PAMM_OK);
                        REQUIRE(cp.total == pamm_compress_workspace(b, n, k, dt) && cp.total > 0);
                        REQUIRE(cp.ncb >= 1 && int64_t(cp.ncb) * 32 * cp.tg >= k && cp.row_tiles * 32 * cp.nw >= b);
                        for (int64_t m : {int64_t(8), int64_t(6144), big}) {
                            pamm::GradPlan gp;
                            REQUIRE(pamm::plan_grad(b, n, k, m, dt, &gp) == PAMM_OK);
                            REQUIRE(gp.total == pamm_grad_workspace(b, n, k, m, dt) && gp.total > 0);
                            REQUIRE(gp.off_bt < gp.total && gp.off_list == 0 && gp.wg_cols >= 1 && gp.chunks >= 1);
                            REQUIRE(int64_t(gp.wg_cols) * 4 * gp.wave_groups * 512 >= m);
                        }
                    }
                }
    }
    REQUIRE(pamm_debug_set_plan(nullptr) == PAMM_OK);
    REQUIRE(pamm_compress_workspace(16, 64, 17, PAMM_BF16) == 0);
    REQUIRE(pamm_compress_workspace(16, 60, 4, PAMM_BF16) == 0);
    REQUIRE(pamm_compress_workspace(16, 64, 4, pamm_dtype(7)) == 0);
    REQUIRE(pamm_grad_workspace(16, 64, 4, 0, PAMM_F32) == 0);
    REQUIRE(pamm_grad_workspace(int64_t(1) << 31, 64, 4, 8, PAMM_F32) == 0);

    // ---- argument checks (fake, never dereferenced addresses)
    const void* A = reinterpret_cast<const void*>(uintptr_t(0x10000));
    const void* odd = reinterpret_cast<const void*>(uintptr_t(0x10004));
    const size_t plenty = size_t(1) << 40;
    pamm::CompressPlan cp;
    pamm::GradPlan gp;
    using namespace pamm;
    REQUIRE(check_compress_args(A, 64, 64, 4, PAMM_BF16, A, A, A, A, plenty, &cp) == PAMM_OK);
    REQUIRE(check_compress_args(nullptr, 64, 64, 4, PAMM_BF16, A, A, A, A, plenty, &cp) == PAMM_ERR_INVALID_ARG);
    REQUIRE(check_compress_args(A, 64, 64, 4, PAMM_BF16, nullptr, A, A, A, plenty, &cp) == PAMM_ERR_INVALID_ARG);
    REQUIRE(check_compress_args(A, 64, 64, 4, PAMM_BF16, A, nullptr, A, A, plenty, &cp) == PAMM_ERR_INVALID_ARG);
    REQUIRE(check_compress_args(A, 64, 64, 4, PAMM_BF16, A, A, nullptr, A, plenty, &cp) == PAMM_ERR_INVALID_ARG);
    REQUIRE(check_compress_args(odd, 64, 64, 4, PAMM_BF16, A, A, A, A, plenty, &cp) == PAMM_ERR_INVALID_ARG);
    REQUIRE(check_compress_args(A, 64, 64, 4, PAMM_BF16, A, A, A, odd, plenty, &cp) == PAMM_ERR_INVALID_ARG);
    REQUIRE(check_compress_args(A, 64, 64, 0, PAMM_BF16, A, A, A, A, plenty, &cp) == PAMM_ERR_INVALID_ARG);
    REQUIRE(check_compress_args(A, 64, 64, 65, PAMM_BF16, A, A, A, A, plenty, &cp) == PAMM_ERR_INVALID_ARG);
    REQUIRE(check_compress_args(A, 0, 64, 4, PAMM_BF16, A, A, A, A, plenty, &cp) == PAMM_ERR_INVALID_ARG);
    REQUIRE(check_compress_args(A, 64, 0, 4, PAMM_BF16, A, A, A, A, plenty, &cp) == PAMM_ERR_INVALID_ARG);
    REQUIRE(check_compress_args(A, 64, 60, 4, PAMM_BF16, A, A, A, A, plenty, &cp) == PAMM_ERR_UNSUPPORTED);
    REQUIRE(check_compress_args(A, 64, 64, 4, pamm_dtype(5), A, A, A, A, plenty, &cp) == PAMM_ERR_UNSUPPORTED);
    REQUIRE(check_compress_args(A, 1 << 20, 64, 20000, PAMM_BF16, A, A, A, A, plenty, &cp) == PAMM_ERR_UNSUPPORTED);
    REQUIRE(check_compress_args(A, 64, 64, 4, PAMM_BF16, A, A, A, nullptr, plenty, &cp) == PAMM_ERR_WORKSPACE);
    REQUIRE(check_compress_args(A, 64, 64, 4, PAMM_BF16, A, A, A, A, 16, &cp) == PAMM_ERR_WORKSPACE);

    REQUIRE(check_contract_args(A, A, A, 64, 4, 64, PAMM_BF16, A, A, plenty, &gp) == PAMM_OK);
    REQUIRE(check_contract_args(nullptr, A, A, 64, 4, 64, PAMM_BF16, A, A, plenty, &gp) == PAMM_ERR_INVALID_ARG);
    REQUIRE(check_contract_args(A, A, A, 64, 65, 64, PAMM_BF16, A, A, plenty, &gp) == PAMM_ERR_INVALID_ARG);
    REQUIRE(check_contract_args(A, A, A, 64, 4, 4, PAMM_BF16, A, A, plenty, &gp) == PAMM_ERR_UNSUPPORTED);
    REQUIRE(check_contract_args(A, A, A, 64, 4, 64, pamm_dtype(-1), A, A, plenty, &gp) == PAMM_ERR_UNSUPPORTED);
    REQUIRE(check_contract_args(A, A, A, 64, 4, 64, PAMM_BF16, A, A, 64, &gp) == PAMM_ERR_WORKSPACE);
    REQUIRE(check_contract_args(A, A, odd, 64, 4, 64, PAMM_BF16, A, A, plenty, &gp) == PAMM_ERR_INVALID_ARG);

    REQUIRE(check_grad_args(A, A, A, A, 64, 64, 4, 64, PAMM_BF16, PAMM_F32, PAMM_DW_N_BY_M, A, A, plenty, &gp) == PAMM_OK);
    REQUIRE(check_grad_args(A, A, A, A, 64, 64, 4, 64, PAMM_BF16, PAMM_BF16, PAMM_DW_M_BY_N, A, A, plenty, &gp) == PAMM_OK);
    REQUIRE(check_grad_args(nullptr, A, A, A, 64, 64, 4, 64, PAMM_BF16, PAMM_F32, PAMM_DW_N_BY_M, A, A, plenty, &gp) == PAMM_ERR_INVALID_ARG);
    REQUIRE(check_grad_args(A, A, A, A, 64, 64, 4, 64, PAMM_BF16, PAMM_F32, PAMM_DW_N_BY_M, nullptr, A, plenty, &gp) == PAMM_ERR_INVALID_ARG);
    REQUIRE(check_grad_args(A, A, A, A, 64, 64, 4, 64, PAMM_BF16, pamm_dtype(2), PAMM_DW_N_BY_M, A, A, plenty, &gp) == PAMM_ERR_UNSUPPORTED);
    REQUIRE(check_grad_args(A, A, A, A, 64, 64, 4, 64, PAMM_BF16, PAMM_F32, pamm_layout(2), A, A, plenty, &gp) == PAMM_ERR_UNSUPPORTED);
    REQUIRE(check_grad_args(A, A, A, A, 64, 64, 4, 12, PAMM_BF16, PAMM_F32, PAMM_DW_N_BY_M, A, A, plenty, &gp) == PAMM_ERR_UNSUPPORTED);
    REQUIRE(check_grad_args(A, A, A, A, 64, 64, 65, 64, PAMM_BF16, PAMM_F32, PAMM_DW_N_BY_M, A, A, plenty, &gp) == PAMM_ERR_INVALID_ARG);
    REQUIRE(check_grad_args(A, A, A, A, 64, 64, 4, 64, PAMM_BF16, PAMM_F32, PAMM_DW_N_BY_M, A, nullptr, plenty, &gp) == PAMM_ERR_WORKSPACE);
    REQUIRE(check_grad_args(A, A, A, A, 64, 64, 4, 64, PAMM_BF16, PAMM_F32, PAMM_DW_N_BY_M, A, A, 1024, &gp) == PAMM_ERR_WORKSPACE);

    // ---- the sketch baseline: planner over ordinary and extreme sizes, argument checks
    for (int64_t b : {int64_t(128), int64_t(700), int64_t(65536), big})
        for (int64_t r : {int64_t(8), int64_t(24), int64_t(72), int64_t(128)})
            for (int64_t m : {int64_t(8), int64_t(6144), big}) {
                pamm::SketchGradPlan sp;
                for (pamm_dtype dt : {PAMM_F32, PAMM_BF16}) {
                    REQUIRE(pamm::plan_sketch_grad(b, 2048, r, m, dt, &sp) == PAMM_OK);
                    REQUIRE(sp.total == pamm_sketch_grad_workspace(b, 2048, r, m, dt) && sp.total > 0);
                    REQUIRE(sp.chunk_rows % 32 == 0 && sp.chunks * sp.chunk_rows >= b && (sp.chunks - 1) * sp.chunk_rows < b);
                    REQUIRE(int64_t(sp.col_groups) * (dt == PAMM_BF16 ? 512 : 256) >= m && sp.nr * 32 >= r && sp.g.kpad >= r &&
                            sp.g.off_bt < sp.total);
                }
            }
    pamm::SketchGradPlan sp;
    REQUIRE(check_sketch_args(A, A, 64, 64, 8, PAMM_BF16, A) == PAMM_OK);
    REQUIRE(check_sketch_args(A, A, 64, 64, 4, PAMM_F32, A) == PAMM_OK);
    REQUIRE(check_sketch_args(A, nullptr, 64, 64, 8, PAMM_BF16, A) == PAMM_ERR_INVALID_ARG);
    REQUIRE(check_sketch_args(A, A, 64, 64, 8, PAMM_BF16, odd) == PAMM_ERR_INVALID_ARG);
    REQUIRE(check_sketch_args(A, A, 4, 64, 8, PAMM_BF16, A) == PAMM_ERR_INVALID_ARG);
    REQUIRE(check_sketch_args(A, A, 64, 64, 12, PAMM_BF16, A) == PAMM_ERR_UNSUPPORTED);
    REQUIRE(check_sketch_args(A, A, 256, 64, 136, PAMM_BF16, A) == PAMM_ERR_UNSUPPORTED);
    REQUIRE(check_sketch_grad_args(A, A, A, 64, 64, 8, 64, PAMM_BF16, A, A, plenty, &sp) == PAMM_OK);
    REQUIRE(check_sketch_grad_args(A, A, A, 64, 64, 8, 64, PAMM_F32, A, A, plenty, &sp) == PAMM_OK);
    REQUIRE(sp.col_groups == 1 && sp.g.kpad == 16);
    REQUIRE(check_sketch_grad_args(A, A, A, 64, 64, 8, 64, pamm_dtype(3), A, A, plenty, &sp) == PAMM_ERR_UNSUPPORTED);
    REQUIRE(check_sketch_grad_args(A, A, nullptr, 64, 64, 8, 64, PAMM_BF16, A, A, plenty, &sp) == PAMM_ERR_INVALID_ARG);
    REQUIRE(check_sketch_grad_args(A, A, A, 64, 64, 8, 12, PAMM_BF16, A, A, plenty, &sp) == PAMM_ERR_UNSUPPORTED);
    REQUIRE(check_sketch_grad_args(A, A, A, 64, 64, 8, 64, PAMM_BF16, A, A, 256, &sp) == PAMM_ERR_WORKSPACE);
    REQUIRE(check_sketch_grad_args(A, A, A, 64, 64, 8, 64, PAMM_BF16, A, nullptr, plenty, &sp) == PAMM_ERR_WORKSPACE);

    double keep = 0.0;
    REQUIRE(keep_of(0.5f, &keep) == PAMM_OK && keep == 0.75);
    REQUIRE(keep_of(1.0f, &keep) == PAMM_OK && keep < 0.0);
    REQUIRE(keep_of(-0.1f, &keep) == PAMM_ERR_INVALID_ARG);
    REQUIRE(keep_of(std::nanf(""), &keep) == PAMM_ERR_INVALID_ARG);

    for (int st = 0; st < 8; ++st) REQUIRE(pamm_status_string(pamm_status(st)) != nullptr);
    for (int id = -1; id <= PAMM_NUM_KERNELS; ++id) REQUIRE(pamm_kernel_name(id) != nullptr);
    std::puts("clean");
    return 0;
}
