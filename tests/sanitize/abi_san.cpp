// Drives the host side of the C ABI - argument validation, option table, the mixed-scheme solvers - in a build
// whose host code is compiled with -fsanitize=address,undefined.  No call here reaches a device: every qp_*
// compute call is refused on the host (that is what is exercised), the solvers are host code.  Values are
// checked by tests/test_abi_host.py and tests/test_msq_host.py; this program only has to run to the end.
// Built and run by tests/test_host_sanitizers.py.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "qp.h"

static void expect(bool ok, const char *what) {
    if (!ok) {
        std::fprintf(stderr, "unexpected status: %s\n", what);
        std::exit(3);
    }
}

int main() {
    expect(qp_version() >= 200, "version");
    for (int c = 0; c < 16; ++c) (void)qp_status_string((qp_status)c);   // (the values an enum of 0 .. 8 can hold)
    // options: every option at its bounds and beyond
    for (int o = -1; o <= QP_OPT_COUNT; ++o) {
        (void)qp_get_option(o);
        for (int v : {-2, -1, 0, 1, 3, 4, 16, 17, 4096, 4097}) (void)qp_set_option(o, v);
    }
    qp_reset_options();
    // descriptors: the legal set and its neighbours
    alignas(256) static unsigned char room[4096];
    for (int scheme = -1; scheme <= 5; ++scheme)
        for (int cb = 0; cb <= 11; ++cb)
            for (int N : {0, 8, 104, 120, 1024, 2048, 14336, 1 << 20})
                for (int layout = 0; layout <= 2; ++layout) {
                    qp_weight w{};
                    w.scheme = scheme; w.M = 48; w.N = N; w.code_bits = cb; w.vec = (scheme == QP_VQ || scheme >= QP_TCQH) ? 2 : 1;
                    w.window_bits = scheme >= QP_TCQ ? 16 : 0; w.tile = scheme >= QP_TCQ ? 256 : 0; w.layout = layout;
                    w.row_stride = 1 << 20; w.codes = room; w.lut = room; w.scales = room;
                    w.tlut_bits = cb <= 8 ? 9 : cb == 9 ? 10 : 11;
                    (void)qp_validate(&w);
                    (void)qp_native_bytes(&w);
                    (void)qp_linear_workspace_bytes(&w, 8);
                    (void)qp_rotate_linear_workspace_bytes(&w, 16);
                    (void)qp_encode_workspace_bytes(&w);
                    // refused before any launch: batch out of range, NULL operands
                    expect(qp_linear(&w, room, 0, 1 << 20, room, 64, nullptr, 0, nullptr) != QP_OK, "linear B = 0");
                    expect(qp_linear(&w, nullptr, 1, 1 << 20, room, 64, nullptr, 0, nullptr) != QP_OK, "linear x = NULL");
                    expect(qp_rotate_linear(&w, room, nullptr, 1024, 1, 1 << 20, room, 64, room, 4096, nullptr) != QP_OK, "rotate signs = NULL");
                    expect(qp_rotate_linear_static(&w, room, (const int8_t *)room, 1024, 17, 1 << 20, room, 64, nullptr) != QP_OK, "static B = 17");
                    expect(qp_dequant(&w, nullptr, nullptr) != QP_OK, "dequant out = NULL");
                    qp_block_item it{&w, room, (const int8_t *)room, 1024, 0, 1 << 20, room, 64};
                    expect(qp_block_enqueue(&it, 1, room, 4096, nullptr) != QP_OK, "block B = 0");
                    qp_block *blk = nullptr;
                    expect(qp_block_create(&it, 1, room, 4096, &blk) != QP_OK && blk == nullptr, "block create B = 0");
                }
    expect(qp_hadamard(room, (const int8_t *)room, 1, 1000, 3, 1000, room, 1000, nullptr) != QP_OK, "hadamard block = 3");
    expect(qp_hadamard(room, (const int8_t *)room, 1, 1024, 1024, 1024, room + 2, 1024, nullptr) != QP_OK, "hadamard overlap");
    expect(qp_bench_stream_read(room, 24, room, nullptr) != QP_OK, "stream bytes % 16");
    (void)qp_kmeans_workspace_bytes(16, 2);
    // the solvers
    {
        const int32_t begin[4] = {0, 2, 5, 6};
        const double loss[6] = {3, 1, 4, 2, 0.5, 7}, cost[6] = {1, 2, 1, 2, 4, 0.25};
        int32_t choice[3];
        double tl = 0, tc = 0;
        for (double budget : {0.1, 3.25, 4.0, 8.25})
            for (int res : {1, 7, 1000, 1 << 22}) (void)qp_msq_solve(3, begin, loss, cost, budget, res, choice, &tl, &tc);
        expect(qp_msq_solve(0, begin, loss, cost, 1.0, 10, choice, nullptr, nullptr) != QP_OK, "msq n = 0");
        expect(qp_msq_solve(3, begin, loss, cost, 1.0, 0, choice, nullptr, nullptr) != QP_OK, "msq resolution = 0");
    }
    for (int nb : {1, 3, 32})
        for (int nq : {1, 4, 16}) {
            std::vector<double> loss((size_t)nb * 7 * nq), cost((size_t)nb * 12 * nq);
            uint32_t s = 99u + nb * 31 + nq;
            auto r = [&]() { s = s * 1664525u + 1013904223u; return 0.25 + (s >> 8) % 1000 / 250.0; };
            for (auto &v : loss) v = r();
            for (auto &v : cost) v = r();
            std::vector<int32_t> assign((size_t)nb * 12);
            double tl, tc;
            for (int fusion = 0; fusion <= 1; ++fusion)
                for (double per_block : {0.5, 6.0, 40.0}) (void)qp_msq_solve_fused(nb, nq, loss.data(), cost.data(), per_block * nb, 4000, fusion, assign.data(), &tl, &tc);
        }
    expect(qp_msq_solve_fused(1, 17, nullptr, nullptr, 1.0, 10, 1, nullptr, nullptr, nullptr) != QP_OK, "fused n_quant = 17");
    std::puts("host side: clean");
    return 0;
}
