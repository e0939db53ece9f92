// Host-side layout and packing code of libelmrnn under AddressSanitizer / UndefinedBehaviorSanitizer.
// Compiled for the host only (no device code, no GPU): every packer writes into a buffer of exactly the
// size its layout function reports, so a write past the end (or before the start) is a sanitizer error;
// the checks below add what a sanitizer cannot see: offsets that overlap, sizes that shrink, values lost.
// Prints "OK <cases>" and exits 0 when everything holds.
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <string>
#include <vector>

#include "internal.h"

using namespace elm;

static long g_cases = 0;
#define REQUIRE(cond)                                                                   \
    do {                                                                                \
        if (!(cond)) {                                                                  \
            std::fprintf(stderr, "FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond);      \
            std::exit(1);                                                               \
        }                                                                               \
    } while (0)

// distinct small integers (exact in float32 and in sums of a few million of them)
static std::vector<float> ramp(size_t n, int start) {
    std::vector<float> v(n);
    for (size_t i = 0; i < n; ++i) v[i] = (float)(1 + (int)((start + i) % 97));
    return v;
}
static double sum_of(const std::vector<float>& v) {
    double s = 0.0;
    for (float x : v) s += x;
    return s;
}
static size_t nonzeros(const std::vector<float>& v) {
    size_t c = 0;
    for (float x : v) c += (x != 0.0f);
    return c;
}

static void dense_cells() {
    const int cells[] = {ELM_CELL_ELMAN, ELM_CELL_LSTM, ELM_CELL_GRU};
    const int Ls[] = {1, 2, 5, 12, 13, 31, 32, 33, 64, 65, 100, 112, 128, 129, 256, 257, 500, 512};
    const int ds[] = {1, 4, 8, 15, 16, 64};
    for (int cell : cells)
        for (int L : Ls)
            for (int d : ds) {
                const int G = gates_of(cell), GL = G * L;
                const std::vector<float> W = ramp((size_t)d * GL, 1), U = ramp((size_t)L * GL, 7), b = ramp(GL, 3);
                const PackedLayout lay = packed_layout(cell, d, L);
                REQUIRE(lay.K == L + d + 1 && lay.KG * 8 >= lay.K && lay.nJB * 32 >= L && lay.R == 8 * lay.KG + 4);
                REQUIRE(lay.floats == lay.copy_floats && lay.floats >= (size_t)lay.nJB * lay.KG * G * 256);
                std::vector<float> out(lay.floats, -1.0f);
                pack_weights(lay, W.data(), U.data(), b.data(), out.data());
                REQUIRE(nonzeros(out) == W.size() + U.size() + b.size());          // every value placed once
                REQUIRE(sum_of(out) == sum_of(W) + sum_of(U) + sum_of(b));
                // spot check of the fragment order: row k, column j of gate g
                const int k = lay.K - 1, j = L - 1, g = G - 1;
                const int kg = k / 8, lane = (j % 32) + 32 * ((k % 8) / 4), e = k % 4, jb = j / 32;
                REQUIRE(out[((((size_t)jb * lay.KG + kg) * G + g) * 64 + lane) * 4 + e] ==
                        U[(size_t)(k - d - 1) * GL + g * L + j]);
                ++g_cases;

                if (tiny_padded_units(cell, L) > 0) {
                    std::vector<float> tiny(tiny_packed_floats(cell, d, L), -1.0f);
                    pack_weights_tiny(cell, d, L, W.data(), U.data(), b.data(), tiny.data());
                    REQUIRE(nonzeros(tiny) == W.size() + U.size() + b.size());
                    REQUIRE(sum_of(tiny) == sum_of(W) + sum_of(U) + sum_of(b));
                    ++g_cases;
                } else {
                    REQUIRE(tiny_packed_floats(cell, d, L) == 0);
                }

                const SplitLayout sl = split_layout(cell, d, L, W.data(), U.data(), b.data());
                REQUIRE(sl.ok == (d <= 15));
                if (sl.ok) {
                    std::vector<unsigned char> packed(sl.bytes, 0xff);
                    pack_weights_split(sl, W.data(), U.data(), b.data(), packed.data());
                    REQUIRE(sl.stride % 16 == 0 && (sl.stride / 16) % 2 == 1 && sl.xoff == sl.KGh * 64);
                    ++g_cases;
                }
            }
    // non-finite weights switch the split mode off instead of being packed
    std::vector<float> W(4, 1.0f), U(16, 1.0f), b(4, 0.0f);
    U[5] = INFINITY;
    REQUIRE(!split_layout(ELM_CELL_ELMAN, 1, 4, W.data(), U.data(), b.data()).ok);
    U[5] = NAN;
    REQUIRE(!split_layout(ELM_CELL_ELMAN, 1, 4, W.data(), U.data(), b.data()).ok);
}

static void multilag_cell() {
    struct Shape { int Q, d, L; };
    // history ring in LDS
    const Shape ring_shapes[] = {{1, 1, 1}, {2, 2, 5}, {10, 4, 100}, {25, 2, 48}, {4, 1, 300}, {3, 64, 64}, {2, 1, 512}};
    for (const Shape& s : ring_shapes) {
        const int ring = s.Q > 1 ? s.Q - 1 : 1;
        const PackedLayout lay = packed_layout(ELM_CELL_FC_MULTILAG, s.d, s.L, ring);
        REQUIRE(lay.K == ring * s.L + s.d + 1 && lay.K <= kFcMaxK && lay.floats == lay.copy_floats * ring);
        const std::vector<float> W = ramp((size_t)s.d * s.L, 1), A = ramp((size_t)s.Q * s.L * s.L, 5), b = ramp(s.L, 2);
        std::vector<float> out(lay.floats, -1.0f);
        pack_weights_fc(lay, W.data(), A.data(), b.data(), out.data());
        // every rotation holds W, b and the lag matrices 1 .. ring once
        const std::vector<float> used(A.begin(), A.begin() + (size_t)ring * s.L * s.L);
        REQUIRE(nonzeros(out) == (size_t)ring * (W.size() + b.size() + used.size()));
        REQUIRE(sum_of(out) == ring * (sum_of(W) + sum_of(b) + sum_of(used)));
        ++g_cases;
    }
    // a launch per step over a history in the caller's workspace
    const Shape step_shapes[] = {{200, 1, 8}, {60, 2, 33}, {14, 1, 100}, {6, 1, 300}, {4, 64, 512}, {50, 4, 100},
                                 {50, 1, 50}, {300, 3, 5}, {130, 1, 10}, {50, 4, 72}, {50, 4, 90}, {3197, 1, 50},
                                 {3197, 1, 100}, {4096, 1, 512}, {64, 64, 96}};
    for (const Shape& s : step_shapes) {
        FcStepLayout lay{};
        REQUIRE(fc_step_layout(s.Q, s.d, s.L, &lay));
        REQUIRE(lay.ring == s.Q - 1 && lay.Lk % 8 == 0 && lay.Lk >= s.L && lay.Lk < s.L + 8);
        REQUIRE(lay.KGpad > lay.KGtot && (int64_t)lay.KGtot * 8 >= (int64_t)lay.ring * lay.Lk + s.d + 1);
        REQUIRE(lay.chunk_rows >= 256 && lay.chunk_rows <= 65536 && lay.chunk_rows % 256 == 0);
        REQUIRE((int64_t)lay.chunk_rows * lay.ring * lay.Lk * 4 < ((int64_t)1 << 31) || lay.chunk_rows == 256);
        REQUIRE(lay.floats == (size_t)lay.nJB * lay.KGpad * 256);
        if (lay.floats <= ((size_t)1 << 27)) {          // pack when the stack is at most 512 MB of host memory
            const std::vector<float> W = ramp((size_t)s.d * s.L, 1), A = ramp((size_t)s.Q * s.L * s.L, 5), b = ramp(s.L, 2);
            const std::vector<float> used(A.begin(), A.begin() + (size_t)lay.ring * s.L * s.L);
            std::vector<float> out(lay.floats, -1.0f);
            pack_weights_fc_steps(lay, W.data(), A.data(), b.data(), out.data());
            REQUIRE(nonzeros(out) == W.size() + b.size() + used.size());
            REQUIRE(sum_of(out) == sum_of(W) + sum_of(b) + sum_of(used));
            REQUIRE((lay.NU > 0) == (s.L > 64 && s.L <= 96));
            if (lay.NU > 0) {
                REQUIRE(lay.floats16 == (size_t)lay.NU * lay.KGpad * 128 && lay.NU * 16 >= s.L);
                std::vector<float> units(lay.floats16, -1.0f);
                pack_weights_fc_rows(lay, W.data(), A.data(), b.data(), units.data());
                REQUIRE(nonzeros(units) == W.size() + b.size() + used.size());
                REQUIRE(sum_of(units) == sum_of(W) + sum_of(b) + sum_of(used));
            }
            ++g_cases;
        }
        // scratch of a call: never smaller for more rows, the two areas do not overlap, whole 256-byte units
        size_t prev = 0;
        const int64_t Ns[] = {1, 255, 256, 257, 4500, 65535, 65536, 65537, 100000, 700000, 4000000};
        for (int64_t N : Ns) {
            const FcScratch sc = fc_scratch(lay, N);
            REQUIRE(sc.pass_rows % 256 == 0 && sc.pass_rows <= lay.chunk_rows && sc.pass_rows >= (N < lay.chunk_rows ? N : lay.chunk_rows));
            REQUIRE(sc.hist_floats == (size_t)sc.pass_rows * lay.ring * lay.Lk);
            REQUIRE(sc.off_sums % 256 == 0 && sc.off_sums >= sc.hist_floats * 4);
            REQUIRE(sc.bytes % 256 == 0 && sc.bytes >= sc.off_sums + sc.sums_floats * 4 && sc.bytes >= prev);
            // what the launcher derives from N stays inside: equal passes of whole 256-row groups
            const int64_t passes = (N + lay.chunk_rows - 1) / lay.chunk_rows;
            const int64_t per_pass = ((N + passes - 1) / passes + 255) / 256 * 256;
            REQUIRE(per_pass <= sc.pass_rows);
            if (lay.nJB <= 2) REQUIRE(sc.sums_floats >= (size_t)per_pass * 128);
            REQUIRE(elm_rnn_hidden_workspace_bytes(ELM_CELL_FC_MULTILAG, N, s.Q, s.d, s.L) == sc.bytes);
            prev = sc.bytes;
            ++g_cases;
        }
    }
    REQUIRE(!fc_step_layout(40000, 1, 512, nullptr));            // a window's history of 8 MiB or more
}

static void solve_plans() {
    const int64_t Ns[] = {1, 33, 64, 127, 2000, 8191, 8192, 100000, 200000, 1000000, 4000000, 50000000};
    const int Ls[] = {1, 5, 10, 31, 32, 33, 100, 128, 256, 288, 289, 500, 512};
    const int ms[] = {1, 2, 4, 5, 16};
    for (int64_t N : Ns)
        for (int L : Ls)
            for (int m : ms)
                for (int forced : {0, 1, 7, 256, 512, 1024}) {
                    const SolvePlan pl = make_solve_plan(N, L, m, forced);
                    const size_t rbytes = (size_t)pl.np * pl.np * sizeof(float);
                    REQUIRE(pl.n == L + m && pl.np % 32 == 0 && pl.np >= pl.n && pl.np < pl.n + 32);
                    REQUIRE(pl.block_rows == 64 || pl.block_rows == 128);
                    REQUIRE(pl.levels >= 1 && pl.levels <= 12 && pl.groups[pl.levels - 1] == 1);
                    REQUIRE(pl.groups[0] >= 1 && pl.groups[0] <= 1024 && (forced == 0 || pl.groups[0] == forced));
                    for (int l = 1; l < pl.levels; ++l) REQUIRE(pl.groups[l] == (pl.groups[l - 1] + 1) / 2);
                    REQUIRE(pl.off_R[0] % 256 == 0 && pl.off_R[1] % 256 == 0 && pl.off_part % 256 == 0 && pl.off_small % 256 == 0);
                    REQUIRE(pl.off_R[0] + rbytes * pl.groups[0] <= pl.off_R[1]);
                    REQUIRE(pl.off_R[1] + rbytes * (pl.levels > 1 ? pl.groups[1] : 1) <= pl.off_part);
                    REQUIRE(pl.off_part + (size_t)1024 * ((size_t)L * m + 2) * sizeof(double) <= pl.off_small);
                    REQUIRE(pl.off_small + SmallArea::doubles(L, m) * sizeof(double) <= pl.bytes);
                    REQUIRE(SmallArea::grad(L, m) == (size_t)L * m && SmallArea::scal(L, m) + 8 == SmallArea::doubles(L, m));
                    if (forced == 0) REQUIRE(elm_rnn_solve_workspace_bytes(N, L, m) == pl.bytes);
                    ++g_cases;
                }
    // the public size queries: zero outside the supported range, additive in their parts
    REQUIRE(elm_rnn_solve_workspace_bytes(0, 4, 1) == 0 && elm_rnn_solve_workspace_bytes(10, 513, 1) == 0 &&
            elm_rnn_solve_workspace_bytes(10, 4, 17) == 0);
    const size_t s = elm_rnn_solve_workspace_bytes(3000, 100, 2);
    REQUIRE(elm_rnn_fit_workspace_bytes(ELM_CELL_LSTM, 3000, 50, 4, 100, 2, 0) == s);
    REQUIRE(elm_rnn_fit_workspace_bytes(ELM_CELL_LSTM, 3000, 50, 4, 100, 2, 1) == s + ((size_t)3000 * 100 * 4 + 255) / 256 * 256);
    REQUIRE(elm_rnn_fit_workspace_bytes(ELM_CELL_FC_MULTILAG, 3000, 50, 4, 100, 2, 0) ==
            s + elm_rnn_hidden_workspace_bytes(ELM_CELL_FC_MULTILAG, 3000, 50, 4, 100));
    REQUIRE(elm_rnn_fit_workspace_bytes(99, 3000, 50, 4, 100, 2, 0) == 0);
    REQUIRE(elm_rnn_fit_streamed_workspace_bytes(ELM_CELL_LSTM, 4000000, 100, 8, 512, 2, 1000) >=
            elm_rnn_solve_workspace_bytes(4000000, 512, 2) + (size_t)1024 * 512 * 4);
    REQUIRE(elm_rnn_hidden_workspace_bytes(ELM_CELL_GRU, 1000, 50, 4, 256) == 0);
    REQUIRE(elm_rnn_hidden_workspace_bytes(ELM_CELL_FC_MULTILAG, 1000, 10, 4, 100) == 0);
}

int main(int argc, char** argv) {
    if (argc > 1 && std::string(argv[1]) == "--selftest") {
        // proves that the instrumentation is live: one float past the end of an exact-size buffer, through
        // a packer, must stop the program (the test expects a sanitizer report and a non-zero status)
        const PackedLayout lay = packed_layout(ELM_CELL_ELMAN, 1, 4);
        const std::vector<float> W = ramp(4, 1), U = ramp(16, 7), b = ramp(4, 3);
        std::vector<float> out(lay.floats - 1);
        pack_weights(lay, W.data(), U.data(), b.data(), out.data());
        std::printf("selftest wrote past the end unnoticed\n");
        return 0;
    }
    dense_cells();
    multilag_cell();
    solve_plans();
    std::printf("OK %ld\n", g_cases);
    return 0;
}
