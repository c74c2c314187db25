// Host-only checks of the planner's integer logic and of the C oracle, meant to run under
// AddressSanitizer and UndefinedBehaviorSanitizer (no GPU, no HIP): every shape the kernels
// rely on is derived here from the planner's output and checked against the buffer sizes.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "plan.hpp"

extern "C" int nvrar_oracle_allreduce(const void *const *in, void *const *out, int G, int N, size_t n, int dtype, int threads);

static int failures = 0;
#define CHECK(cond) do { if (!(cond)) { ++failures; std::fprintf(stderr, "line %d: %s (P=%d G=%d n=%zu dtype=%d)\n", __LINE__, #cond, P, G, n, dtype); } } while (0)

static void check_shape(int P, int G, size_t n, int dtype) {
    rar_plan_t *plan = nullptr;
    if (rar_plan(P, G, n, dtype, &plan) != RAR_OK) { ++failures; return; }
    const rar::Geometry &g = plan->geo;
    // chunks tile [0, n) in order, start on 16-byte groups
    size_t pos = 0;
    for (int c = 0; c < G; ++c) {
        size_t off = 0, len = 0;
        CHECK(rar_plan_chunk(plan, c, &off, &len) == RAR_OK);
        CHECK(off == pos);
        CHECK(len == 0 || off % g.per_vec == 0);
        CHECK(len <= g.chunk_len);
        pos = off + len;
    }
    CHECK(pos == n);
    CHECK(g.chunk_stride >= g.chunk_vecs * 16 && g.chunk_stride % 256 == 0);
    CHECK(g.flags_bytes >= static_cast<size_t>(g.L + 1) * P * rar::kMaxWorkgroupsPerRank * 4);
    CHECK(g.N == (1 << g.L) + g.fold && g.fold >= 0 && g.fold < (1 << g.L));
    CHECK(g.packed_levels == (g.packed_offset ? g.L + (g.fold ? 1 : 0) : 0));
    CHECK(g.data_offset % 256 == 0);
    CHECK(g.scratch_bytes >= g.data_offset + static_cast<size_t>(g.L + 1) * P * g.chunk_stride);
    CHECK(g.fused_bytes == g.data_offset + static_cast<size_t>(g.L + 1) * P * g.chunk_stride);
    // the second set of exchange buffers (odd calls of a chain) exists exactly where the data+flag
    // buffers do, lies behind them, and has the shape of the first set
    CHECK((g.alt_offset != 0) == (g.packed_offset != 0) && (g.packed_alt_offset != 0) == (g.packed_offset != 0));
    if (g.alt_offset) {
        CHECK(g.alt_offset == g.packed_offset + static_cast<size_t>(g.packed_levels) * P * g.packed_stride);
        CHECK(g.packed_alt_offset == g.alt_offset + static_cast<size_t>(g.L + 1) * P * g.chunk_stride);
        CHECK(g.scratch_bytes == g.packed_alt_offset + static_cast<size_t>(g.packed_levels) * P * g.packed_stride);
        CHECK(g.alt_offset % 256 == 0 && g.packed_alt_offset % 256 == 0);
    }
    // peers: mutual, same local id; a node that sits out has a partner on the next node that
    // takes part, and nothing reaches past rank P - 1
    for (int p = 0; p < P; ++p) {
        const int partner = rar_plan_fold_partner(plan, p);
        CHECK(partner >= 0 && partner < P && partner % G == p % G);
        CHECK(rar_plan_fold_partner(plan, partner) == p);
        const bool idle = rar::sits_out(p / G, g.fold);
        CHECK(!idle || partner == p + G);
        CHECK(!rar::folds_in(p / G, g.fold) || partner == p - G);
        for (int l = 0; l < g.L; ++l) {
            const int q = rar_plan_peer(plan, p, l);
            if (idle) { CHECK(q == p); continue; }
            CHECK(q >= 0 && q < P && q % G == p % G && rar_plan_peer(plan, q, l) == p && q != p);
            CHECK(!rar::sits_out(q / G, g.fold));
        }
    }
    // every tuning the launchers can see keeps all accesses inside the buffers
    const long resident_cases[3][4] = {{0, 0, 0, 0}, {2048, 2048, 1024, 512}, {256, 256, 256, 256}};
    const size_t C_values[5] = {0, 4096, 8192, 16384, 32768};
    const int B_values[6] = {0, 1, 3, 16, 100, 256};
    for (const auto &resident : resident_cases)
        for (size_t C_s : C_values)
            for (int B_s : B_values) {
                CHECK(rar_plan_set_tuning(plan, B_s, C_s) == RAR_OK);
                const rar::Tuning t = rar::resolve_tuning(*plan, resident[0] ? resident : nullptr);
                CHECK(t.B_s >= 1 && t.B_s <= rar::kMaxWorkgroupsPerRank && t.iters >= 1);
                CHECK(t.unroll == 1 || t.unroll == 2 || t.unroll == 4 || t.unroll == 8);
                const size_t slice = static_cast<size_t>(rar::kThreads) * t.unroll;
                // all slices are covered
                CHECK(static_cast<size_t>(t.B_s) * t.iters * slice >= g.chunk_vecs);
                // vector indices stay 32-bit
                CHECK((static_cast<size_t>(t.B_s) * t.iters + 1) * slice < (static_cast<size_t>(1) << 32));
                // ring reuse (three or more trips) fits inside a partial buffer
                if (t.iters >= 3) CHECK(2 * static_cast<size_t>(t.B_s) * slice * 16 <= g.chunk_stride);
                // packed words of the last slice that holds data stay inside a packed buffer
                if (g.packed_offset) {
                    const size_t slices_with_data = (g.chunk_vecs + slice - 1) / slice;
                    CHECK(slices_with_data * slice * 32 <= g.packed_stride);
                    CHECK(g.scratch_bytes >= g.packed_offset + static_cast<size_t>(g.packed_levels) * P * g.packed_stride);
                }
                if (resident[0]) {
                    const int idx = t.unroll == 1 ? 0 : t.unroll == 2 ? 1 : t.unroll == 4 ? 2 : 3;
                    CHECK(static_cast<long>(P) * t.B_s <= resident[idx] || t.B_s == 1);
                }
                // never more than four workgroups per compute unit (256 units until a device is known)
                CHECK(static_cast<long>(P) * t.B_s <= 4L * 256 || t.B_s == 1);
                // a chained launch: the same, and without a second set of buffers two places per
                // workgroup fit inside one partial buffer
                const rar::Tuning tc = rar::resolve_chain_tuning(*plan, resident[0] ? resident : nullptr);
                CHECK(tc.unroll == t.unroll && tc.B_s >= 1 && tc.B_s <= t.B_s && tc.iters >= 1);
                CHECK(static_cast<size_t>(tc.B_s) * tc.iters * slice >= g.chunk_vecs);
                if (g.L > 0 && g.alt_offset == 0) {
                    CHECK(2 * static_cast<size_t>(tc.B_s) * slice * 16 <= g.chunk_stride);
                    CHECK(tc.iters >= 2);
                }
            }
    rar_plan_free(plan);
}

static void check_oracle(int P, int G, size_t n, int dtype) {
    const size_t es = dtype == 0 ? 2 : 4;
    std::vector<std::vector<unsigned char>> in(P, std::vector<unsigned char>(n * es)), out(P, std::vector<unsigned char>(n * es));
    std::vector<const void *> ip(P);
    std::vector<void *> op(P);
    uint32_t state = 12345u + P * 7 + G;
    for (int p = 0; p < P; ++p) {
        for (size_t i = 0; i < n; ++i) {
            state = state * 1664525u + 1013904223u;
            const float f = (static_cast<float>(state >> 8) / 8388608.0f - 1.0f);
            uint32_t u; std::memcpy(&u, &f, 4);
            if (dtype == 0) { uint16_t h = static_cast<uint16_t>(u >> 16); std::memcpy(&in[p][i * 2], &h, 2); }
            else std::memcpy(&in[p][i * 4], &f, 4);
        }
        ip[p] = in[p].data();
        op[p] = out[p].data();
    }
    if (nvrar_oracle_allreduce(ip.data(), op.data(), G, P / G, n, dtype, 1) != 0) { ++failures; return; }
    for (int p = 1; p < P; ++p) CHECK(std::memcmp(out[p].data(), out[0].data(), n * es) == 0);
}

int main() {
    const int Gs[] = {1, 2, 3, 4, 5, 8};
    const size_t ns[] = {1, 7, 8, 9, 63, 64, 65, 1000, 4096, 65536, 65537, 1048576, 33554432, 100000007};
    for (int G : Gs)
        for (int N = 1; N * G <= RAR_MAX_RANKS; N = N < 8 ? N + 1 : N < 16 ? N + 3 : N * 2 - 5)
            for (size_t n : ns)
                for (int dtype = 0; dtype < 2; ++dtype) check_shape(N * G, G, n, dtype);
    for (int G : Gs)
        for (int N = 1; N <= 9 && N * G <= 36; ++N)
            for (size_t n : {size_t(1), size_t(7), size_t(33), size_t(1001)})
                for (int dtype = 0; dtype < 2; ++dtype) check_oracle(N * G, G, n, dtype);
    std::printf(failures ? "host checks FAILED: %d\n" : "host checks ok\n", failures);
    return failures ? 1 : 0;
}
