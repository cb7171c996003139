// Host-side check of the launch plans and workspace layouts (csrc/plan.hpp): built and run by
// tests/test_plan_host.py with the host compiler; prints one line per violated invariant and, per
// shape, the workspace size the layouts need (compared with mage_workspace_bytes by the test).
#include <cstdio>
#include <cstdint>
#include <initializer_list>

#include "../paper_2602_14209_amd/csrc/plan.hpp"

using namespace mage;

static int failures = 0;
#define CHECK(cond, ...) do { if (!(cond)) { ++failures; std::printf("FAIL %s:", #cond); std::printf(__VA_ARGS__); std::printf("\n"); } } while (0)

static void check_dense(const char *what, const mage_shape &s, const SplitPlan &p, bool rows_in_one)
{
    const long long L = s.L;
    CHECK(p.tile > 0 && p.kps >= p.tile && p.kps % p.tile == 0, " %s L=%lld kps=%d", what, L, p.kps);
    CHECK(p.n_split >= 1 && p.n_cyc == p.n_split, " %s L=%lld n_split=%d n_cyc=%d", what, L, p.n_split, p.n_cyc);
    CHECK((long long)p.n_split * p.kps >= L, " %s L=%lld: keys not covered", what, L);
    CHECK((long long)(p.n_split - 1) * p.kps < L, " %s L=%lld: an empty split", what, L);
    CHECK(p.blk_split >= 0 && p.blk_split < p.n_split, " %s blk_split=%d", what, p.blk_split);
    CHECK(p.rpad >= p.R && p.row_groups * p.rows_per_wg == p.rpad, " %s rows R=%d rpad=%d", what, p.R, p.rpad);
    // tiles dealt round-robin: split s < n_cyc owns tiles s, s + n_cyc, ...; every tile exactly once
    const long long tiles = (L + p.tile - 1) / p.tile;
    long long owned = 0;
    for (int sp = 0; sp < p.n_cyc; ++sp) owned += tiles > sp ? (tiles - sp + p.n_cyc - 1) / p.n_cyc : 0;
    CHECK(owned == tiles, " %s L=%lld: %lld of %lld tiles owned", what, L, owned, tiles);
    (void)rows_in_one;
}

template <class Layout>
static void check_offsets(const char *what, std::initializer_list<size_t> offs, size_t bytes)
{
    size_t prev = 0;
    bool first = true;
    for (size_t o : offs) {
        CHECK(o % 256 == 0, " %s offset %zu not 256-aligned", what, o);
        CHECK(first || o > prev, " %s offsets not increasing (%zu after %zu)", what, o, prev);
        prev = o;
        first = false;
    }
    CHECK(bytes >= prev, " %s total %zu < last offset %zu", what, bytes, prev);
}

int main()
{
    for (int dt : {MAGE_F32, MAGE_BF16})
        for (int Hkv : {1, 2, 4, 8})
            for (int G : {1, 4, 7})
                for (int B : {1, 5, 32, 48})
                    for (int d : {64, 128})
                        for (long long L : {1LL, 63LL, 64LL, 65LL, 1000LL, 8192LL, 65536LL, 131073LL, 1LL << 20}) {
                            for (long long k : {1LL, L < 512 ? L : 512LL, L}) {
                                if (k > (1 << 20)) continue;
                                mage_shape s{B, Hkv * G, Hkv, d, (int64_t)L, (int)k, (mage_dtype)dt};
                                const SplitPlan pd = plan_dense(s), ps = plan_stats(s), pc = plan_colsum(s), pp = plan_sparse(s);
                                check_dense("dense", s, pd, false);
                                check_dense("stats", s, ps, false);
                                check_dense("colsum", s, pc, true);
                                CHECK(pp.kps % pp.tile == 0 && (long long)pp.n_cyc * pp.kps >= k, " sparse k=%lld n_cyc=%d kps=%d", k, pp.n_cyc, pp.kps);
                                CHECK(pp.blk_split >= 0 && pp.blk_split < pp.n_split, " sparse blk_split=%d of %d", pp.blk_split, pp.n_split);
                                const SelectLayout sl = select_layout(s, ps);
                                check_offsets<SelectLayout>("select", {sl.part_m, sl.part_l, sl.lse2, sl.alpha, sl.gmax}, sl.bytes);
                                const Step1Layout tl = step1_layout(s, pd);
                                check_offsets<Step1Layout>("step1", {tl.partials, tl.stat_m, tl.stat_l, tl.lse2, tl.alpha, tl.gmax}, tl.bytes);
                                size_t need = partial_bytes(s, pd);
                                if (partial_bytes(s, pp) > need) need = partial_bytes(s, pp);
                                if (sl.bytes > need) need = sl.bytes;
                                if (tl.bytes > need) need = tl.bytes;
                                std::printf("NEED %d %d %d %d %lld %lld %d %zu\n", B, Hkv * G, Hkv, d, L, k, dt, need);
                            }
                        }
    std::printf(failures ? "FAILED %d\n" : "OK\n", failures);
    return failures ? 1 : 0;
}
