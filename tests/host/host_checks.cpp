// Host-only checks of the library's argument validation, size arithmetic, split planning and the multiply-shift
// division, built with AddressSanitizer and UndefinedBehaviorSanitizer by tests/test_host_sanitize.py (no GPU code runs).
#include "../../paper_2411_00288_amd/csrc/ss_conv_params.h"
#include <cstdio>
#include <cstdlib>

using namespace ss;

static int failures = 0;
#define CHECK(c) do { if (!(c)) { std::printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #c); failures++; } } while (0)

static ss_weight_desc desc(int cout, int cin, int kh, int kw, int dtype = SS_F16, int korder = SS_K_CRS)
{
    ss_weight_desc d{cout, cin, kh, kw, dtype, korder};
    return d;
}

// floor(n / d) as the kernels compute it from the host-side constants
static unsigned fast_div_host(unsigned n, unsigned mul, unsigned sh) { return (unsigned)(((unsigned long long)n * mul) >> sh); }

int main()
{
    // ---- descriptor validation and sizes
    ss_weight_desc d = desc(256, 256, 3, 3);
    CHECK(check_desc(&d, true) == SS_OK);
    CHECK(check_desc(nullptr, true) == SS_ERR_INVALID_ARG);
    TileDims t = tile_dims(&d);
    CHECK(t.K == 2304 && t.G == 576 && t.Mt == 8 && t.Ks == 72 && t.Kp == 36);
    CHECK(packed_size(t) == 256u + 256u * 2304u + 256u * 2304u / 8u);
    CHECK(dense_size(t) == 256u + 2u * 256u * 2304u);
    ss_weight_desc stem = desc(64, 3, 7, 7);
    CHECK(check_desc(&stem, true) == SS_ERR_UNSUPPORTED && check_desc(&stem, false) == SS_OK);
    for (int bad = 0; bad < 4; bad++) {
        ss_weight_desc b = desc(bad == 0 ? 0 : 8, bad == 1 ? -1 : 8, 1, 1, bad == 2 ? 9 : SS_F16, bad == 3 ? 7 : SS_K_CRS);
        CHECK(check_desc(&b, false) == SS_ERR_INVALID_ARG);
    }
    ss_weight_desc huge = desc(1 << 20, 1 << 12, 3, 3);
    CHECK(check_desc(&huge, true) == SS_ERR_UNSUPPORTED);
    ss_weight_desc q = desc(40, 8, 3, 3, SS_I8);
    CHECK(tile_dims(&q).Ks == 2 && tile_dims(&q).Kp == 2);

    // ---- multiply-shift division: exact for every numerator the kernels can form
    // all divisors up to 4096 on a dense set of numerators, and sampled large divisors up to 2^31 - 1 at their multiples +- 1
    for (unsigned dv = 1; dv <= 4096; dv++) {
        unsigned mul, sh;
        fast_div_setup(dv, &mul, &sh);
        for (unsigned n = 0; n < 70000u; n += (dv < 64 ? 1 : 7)) CHECK(fast_div_host(n, mul, sh) == n / dv);
        for (unsigned long long m = 1; m * dv < (1ull << 31); m = m * 3 + 1) {
            const unsigned n = (unsigned)(m * dv);
            CHECK(fast_div_host(n, mul, sh) == n / dv && fast_div_host(n - 1, mul, sh) == (n - 1) / dv);
            if (n + 1 < (1u << 31)) CHECK(fast_div_host(n + 1, mul, sh) == (n + 1) / dv);
        }
        CHECK(fast_div_host((1u << 31) - 1, mul, sh) == ((1u << 31) - 1) / dv);
    }
    unsigned long long state = 88172645463325252ull;
    for (int i = 0; i < 2000000; i++) {
        state ^= state << 13; state ^= state >> 7; state ^= state << 17;
        unsigned dv = (unsigned)(state >> 33) | 1u;                 // odd, < 2^31
        unsigned n = (unsigned)(state & 0x7FFFFFFFu);
        unsigned mul, sh;
        fast_div_setup(dv, &mul, &sh);
        CHECK(fast_div_host(n, mul, sh) == n / dv);
    }

    // ---- tile choice and split planning stay inside their ranges for every layer-like shape
    for (int cout : {8, 64, 96, 128, 200, 256, 512, 1024, 2048})
        for (int cin : {32, 64, 96, 256, 512, 2048})
            for (int k : {1, 3})
                for (long long P : {1ll, 49ll, 392ll, 3136ll, 12544ll, 200704ll, 802816ll})
                    for (int forced_tile : {-1, 0, 3, 5, 10})
                        for (int forced_split : {0, 1, 3, 64}) {
                            ss_weight_desc w = desc(cout, cin, k, k, SS_BF16);
                            const int Ks = tile_dims(&w).Ks;
                            SplitPlan pl = plan_split(&w, P, Ks, 256, forced_tile, forced_split);
                            CHECK(pl.nsplit >= 1);
                            if (pl.nsplit > 1) {
                                const int ksteps = k == 3 ? 9 : 4;
                                CHECK(pl.nsplit <= (Ks + ksteps - 1) / ksteps);
                                CHECK(pl.tile >= 0 && pl.tile <= 5 && pl.bn == 64 && (pl.bm == 64 || pl.bm == 128 || pl.bm == 256));
                                CHECK(pl.tiles == (long long)((cout + pl.bm - 1) / pl.bm) * ((P + 63) / 64));
                                CHECK(pl.ctr_bytes % 256 == 0 && pl.ctr_bytes >= (size_t)pl.tiles * 4);
                                CHECK(pl.part_bytes == (size_t)pl.tiles * pl.nsplit * pl.bm * pl.bn * 4);
                                if (forced_split == 0) CHECK(pl.tiles * pl.nsplit <= 256 && pl.ctr_bytes + pl.part_bytes <= ((size_t)16 << 20) + ((size_t)64 << 10));
                            }
                        }
    ss_weight_desc i8 = desc(512, 512, 3, 3, SS_I8);
    CHECK(plan_split(&i8, 49, tile_dims(&i8).Ks, 256, -1, 4).nsplit == 1);      // 8-bit operands never split
    if (failures == 0) std::printf("host checks passed\n");
    return failures ? 1 : 0;
}
