// Host-side harness run under -fsanitize=address,undefined by tests/test_sanitizers.py: table construction
// and packing for every data type, and the launch plan with the unit geometry for element counts on both
// sides of 2^32.  Exits 0 when every check holds; prints the first failure otherwise.
#include <cstdio>
#include <cstdlib>
#include <memory>
#include <vector>

#include "dq8_plan.hpp"
#include "dq8_tables.hpp"
#include "dq8_units.hpp"

static int failures = 0;
#define CHECK(cond, ...)                                  \
    do {                                                  \
        if (!(cond)) {                                    \
            if (failures++ < 20) {                        \
                std::printf("FAIL %s: ", #cond);          \
                std::printf(__VA_ARGS__);                 \
                std::printf("\n");                        \
            }                                             \
        }                                                 \
    } while (0)

static void check_tables()
{
    for (int kind = 0; kind < 4; ++kind) {
        std::unique_ptr<dq8::Tables> t(new dq8::Tables);
        const int rc = dq8::build_tables(kind, t.get());
        CHECK(rc == 0, "kind %d status %d", kind, rc);
        std::vector<uint32_t> words(dq8::kTableWords);  // exactly sized: an overrun is an address error
        dq8::pack_tables(*t, words.data());
        CHECK(words[dq8::kNBucketOff] == t->n_bucket && t->n_bucket <= (uint32_t)dq8::kBucketCapacity,
              "kind %d bucket count %u", kind, t->n_bucket);
        CHECK(t->n_mag >= 2 && t->n_mag <= 128, "kind %d magnitudes %u", kind, t->n_mag);
        for (uint32_t r = 1; r < t->n_mag; ++r) CHECK(t->cb[t->canon[r]] > t->cb[t->canon[r - 1]], "kind %d rank %u", kind, r);
    }
    dq8::Tables t;
    CHECK(dq8::build_tables(4, &t) == 2 && dq8::build_tables(-1, &t) == 2, "unknown kinds are rejected");
}

template <int U>
static void check_units(size_t n, size_t block)
{
    for (int wpc : {3, 8, 32}) {
        const Plan p = make_plan(n, block, 256, wpc, 1, kWavesPerWg, (size_t)U);
        const size_t B = block_length(n, block);
        CHECK(p.B == B && p.nb == (n + B - 1) / B && p.upb == (B + U - 1) / U, "n %zu block %zu", n, block);
        CHECK(p.n_units >= 1 && p.n_teams >= 1 && p.grid >= 1, "n %zu block %zu", n, block);
        // every team walks ceil(units / teams) units at most and no team is left without one
        const size_t per = (p.n_units + p.n_teams - 1) / p.n_teams;
        CHECK((per - 1) * p.n_teams < p.n_units, "n %zu block %zu: %zu units on %zu teams", n, block, p.n_units, p.n_teams);
        // units: the leading and the trailing ones, and the ones around element 2^32
        std::vector<size_t> probes;
        auto window = [&](size_t centre) {
            const size_t lo = centre > 600 ? centre - 600 : 0, hi = centre + 600 < p.n_units ? centre + 600 : p.n_units;
            for (size_t u = lo; u < hi; ++u) probes.push_back(u);
        };
        if (p.n_units <= 200000) {
            for (size_t u = 0; u < p.n_units; ++u) probes.push_back(u);
        } else {
            window(0);
            window(p.n_units - 1);
            if (n > ((size_t)1 << 32)) window((size_t)((double)p.n_units * (double)((size_t)1 << 32) / (double)n));
            window(p.n_units / 3);
        }
        size_t prev_u = (size_t)-2, prev_end = 0;
        for (size_t u : probes) {
            const Unit un = unit_of<U>(u, n, p.B, p.nb, p.upb);
            CHECK(un.len >= 1 && un.len <= (uint32_t)U, "unit %zu of n %zu block %zu: length %u", u, n, block, un.len);
            CHECK(un.start < n && un.start + un.len <= n, "unit %zu of n %zu block %zu: [%zu, +%u)", u, n, block, un.start, un.len);
            CHECK(un.block == un.start / B && (un.start + un.len - 1) / B == un.block, "unit %zu crosses a block", u);
            if (u == 0) CHECK(un.start == 0, "the first unit starts at %zu", un.start);
            if (u == prev_u + 1) CHECK(un.start == prev_end, "unit %zu starts at %zu, the one before ended at %zu", u, un.start, prev_end);
            if (u + 1 == p.n_units) CHECK(un.start + un.len == n, "the last unit ends at %zu of %zu", un.start + un.len, n);
            prev_u = u;
            prev_end = un.start + un.len;
        }
    }
}

static void check_plans()
{
    const size_t two32 = (size_t)1 << 32;
    const size_t sizes[] = {1, 3, 255, 256, 4096, 4097, 61100840, two32 - 1, two32, two32 + 12305, 3 * (two32 / 2) + 1,
                            ((size_t)1 << 40) + 5};
    const size_t blocks[] = {0, 1, 4, 100, 1000, 4096, 5000, 16384, 65536, two32 + 7};
    for (size_t n : sizes)
        for (size_t b : blocks) {
            if (b == 1 && n > 1000000) continue;  // one unit per element: covered by the small sizes
            check_units<256>(n, b);
            check_units<1024>(n, b);
            check_units<4096>(n, b);
        }
    // teams of one to four wavefronts (twelve wavefronts per workgroup), a block of up to W x 1024 elements per team
    for (int W = 1; W <= 4; ++W)
        for (size_t b : {(size_t)(W * 1024), (size_t)(W * 1024 - 24), (size_t)((W - 1) * 1024 + 4)})
            for (size_t n : {b, 5 * b + 3, (size_t)61100840, two32 + 12305}) {
                const Plan p = make_plan(n, b, 256, 12, W, 12, kUnit);
                CHECK(p.upb == 1 && p.n_units == p.nb, "team plan: n %zu block %zu", n, b);
                CHECK(p.n_teams == (size_t)p.grid * (size_t)(12 / W) && p.n_teams <= (size_t)256 * 12 / W + 12, "team plan: n %zu block %zu W %d", n, b, W);
                const size_t per = (p.n_units + p.n_teams - 1) / p.n_teams;
                CHECK((per - 1) * p.n_teams < p.n_units, "team plan: %zu units on %zu teams", p.n_units, p.n_teams);
                const Unit un = unit_of<kUnit>(p.nb - 1, n, p.B, p.nb, 1);
                CHECK(un.block == p.nb - 1 && un.start == (p.nb - 1) * b && un.start + un.len == n && un.len <= (uint32_t)(W * 1024),
                      "team plan: last unit of n %zu block %zu", n, b);
            }
    // tensors back to back: units of 1024 elements, items of one or four units, sixteen wavefronts per workgroup
    for (size_t n : {(size_t)1, (size_t)1023, (size_t)1024, (size_t)1025, (size_t)1863690, (size_t)61100840, two32 + 12305})
        for (int wpc : {16, 32})
            for (bool grouped : {false, true}) {
                const SegPlan p = make_segment_plan(256, n, 17, wpc, grouped);
                CHECK(p.n_units == (n + 1023) / 1024 && (p.group == 1 || (grouped && p.group == 4)), "segment plan of %zu", n);
                CHECK(p.n_items * p.group >= p.n_units && (p.n_items - 1) * p.group < p.n_units, "segment plan of %zu: items", n);
                CHECK(p.grid >= 1 && p.n_waves == (size_t)p.grid * kSegWaves && p.n_waves < p.n_items + kSegWaves, "segment plan of %zu: grid", n);
                CHECK(p.n_waves <= (size_t)256 * 32 && p.lds == 18 * sizeof(uint64_t), "segment plan of %zu: size", n);
                CHECK(p.group == 1 || p.n_items >= 2 * p.n_waves, "segment plan of %zu: too few items of four", n);
            }
    for (int K = 0; K <= DQ8_MAX_K; ++K) {
        const int c = chunk_size(K);
        CHECK(c >= 1 && c <= 8, "chunk of %d workers: %d", K, c);
    }
    for (size_t b : {(size_t)1, (size_t)255, (size_t)256, (size_t)257, (size_t)4096, (size_t)4097, (size_t)16384, (size_t)16385}) {
        const size_t h = holding_unit(b), e = encode_unit(b, true);
        CHECK(h >= 256 && h <= 4096 && (h & (h - 1)) == 0 && (h >= b || h == 4096), "holding unit of %zu: %zu", b, h);
        CHECK(e >= h && e <= 16384, "encode unit of %zu: %zu", b, e);
        int q = 16, w = 4;
        fit_unit_to_block(b, &q, &w);
        CHECK(q >= 1 && q <= 16 && w >= 4 && w <= 32 && ((size_t)q * 256 <= b || q == 1), "unit fitted to %zu: %d quads", b, q);
    }
    for (size_t n : {(size_t)0, (size_t)1023, (size_t)1024, two32 + 1024 * 7 + 3}) {
        const SmallPlan sp = make_small_plan(n, 256, 32, 4);
        CHECK(sp.done <= n && sp.done == sp.n_units * kSmallUnit && n - sp.done < kSmallUnit, "small plan of %zu", n);
        CHECK(sp.n_units == 0 || sp.n_waves * ((sp.n_units + sp.n_waves - 1) / sp.n_waves) >= sp.n_units, "small plan of %zu", n);
    }
}

int main()
{
    check_tables();
    check_plans();
    if (failures) {
        std::printf("%d checks failed\n", failures);
        return 1;
    }
    std::printf("host checks ok\n");
    return 0;
}
