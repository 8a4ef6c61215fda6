// Host-only driver for the library's index arithmetic, sort keys, workspace layout and pair
// test (csrc/nms_host_logic.h, csrc/nms_pair.h), built with a plain host compiler by
// tests/test_host_logic.py.  No GPU, no HIP.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../paper_2502_00535_amd/csrc/nms_host_logic.h"

template <int kSuper>
static long long sweep_units(long long limit)
{
    // the numbering by construction: super-row sr holds kSuper * (sr + 1) units, tc = 0, 1, ...
    int want_sr = 0, want_tc = 0;
    for (long long g = 0; g < limit; ++g) {
        int sr = -1, tc = -1;
        nms_triangle_unit<kSuper>((int)g, sr, tc);
        if (sr != want_sr || tc != want_tc) return g;
        if (++want_tc == kSuper * (want_sr + 1)) {
            want_tc = 0;
            ++want_sr;
        }
    }
    return -1;
}

static int count_units_by_hand(int T, int super)
{
    int total = 0;
    for (int sr = 0; sr * super < T; ++sr) {
        const int last_row = (sr + 1) * super < T ? (sr + 1) * super : T;  // tile rows of the super-row end here
        total += last_row;                                                  // tc = 0 .. last_row - 1
    }
    return total;
}

int main(int argc, char **argv)
{
    if (argc < 2) return 2;
    if (!strcmp(argv[1], "triangle")) {
        const long long limit = atoll(argv[2]);
        const long long bad1 = sweep_units<1>(limit), bad2 = sweep_units<2>(limit), bad4 = sweep_units<4>(limit);
        printf("first_mismatch %lld %lld %lld\n", bad1, bad2, bad4);
        int wrong = 0;
        for (int T = 0; T <= 1100; ++T)
            for (int super : {1, 2, 4})
                if (nms_triangle_units(T, super) != count_units_by_hand(T, super)) ++wrong;
        printf("unit_count_mismatches %d\n", wrong);
        // the last unit of every count maps inside the triangle
        int outside = 0;
        for (int T = 1; T <= 1100; ++T) {
            int sr, tc;
            nms_triangle_unit<4>(nms_triangle_units(T, 4) - 1, sr, tc);
            if (sr != (T - 1) / 4 || tc != T - 1) ++outside;
            nms_triangle_unit<1>(nms_triangle_units(T, 1) - 1, sr, tc);
            if (sr != T - 1 || tc != T - 1) ++outside;
        }
        printf("last_unit_mismatches %d\n", outside);
        return 0;
    }
    if (!strcmp(argv[1], "shares")) {
        // every batch shape that the small-frames kernels take: the share of a workgroup must fit the kernel's tables
        // (one victim per thread: 512 threads up to 512 boxes per frame, 1024 beyond), no workgroup beyond the frame's tiles
        long long taken = 0, bad = 0;
        for (int n_max = 1; n_max <= 4200; ++n_max) {
            for (int frames = 1; frames <= 70000; frames = frames < 600 ? frames + 1 : frames * 2 + 1) {
                if (!nms_use_small_frames(n_max, frames)) continue;
                ++taken;
                const int tiles = (n_max + 63) / 64;
                const int parts = nms_small_frames_parts(frames, n_max);
                const int share_tiles = (tiles + parts - 1) / parts;
                const int threads = n_max <= 512 ? 512 : 1024;
                const bool ok = n_max > 448 && n_max <= 4096 && parts >= 1 && parts <= 64 && parts <= tiles &&
                                share_tiles * 64 <= threads && (long long)frames * parts <= 2147483647ll &&
                                nms_route_for(n_max, frames, 4096) == kNmsRouteSmallFrames;
                if (!ok) {
                    if (!bad) printf("first_bad %d %d parts %d\n", n_max, frames, parts);
                    ++bad;
                }
            }
        }
        printf("taken %lld bad %lld\n", taken, bad);
        return 0;
    }
    if (!strcmp(argv[1], "layout")) {
        int n_max, frames, chunk;
        while (scanf("%d %d %d", &n_max, &frames, &chunk) == 3) {
            const int n_pad = (n_max + 63) / 64 * 64;
            const NmsRunLayout l = nms_run_layout(n_max, n_pad, frames, chunk);
            printf("%zu %zu %zu %zu %zu %zu %zu %zu\n", l.order, l.sorted5, l.ysc, l.ytile, l.tsc, l.keys, l.stage, l.end);
        }
        return 0;
    }
    if (!strcmp(argv[1], "keys")) {
        FILE *f = fopen(argv[2], "rb");
        if (!f) return 3;
        std::vector<float> s;
        float v;
        while (fread(&v, sizeof v, 1, f) == 1) s.push_back(v);
        fclose(f);
        for (size_t i = 0; i < s.size(); ++i) printf("%016llx\n", nms_rank_key(s[i], (unsigned)i));
        return 0;
    }
    if (!strcmp(argv[1], "pairs")) {
        // records of 9 floats: victim box, outranking box, theta -> "exact fast" decisions (fast = -1 outside its range)
        FILE *f = fopen(argv[2], "rb");
        if (!f) return 3;
        float r[9];
        while (fread(r, sizeof(float), 9, f) == 9) {
            const float area = nms_box_area(r[4], r[5], r[6], r[7]);
            const int exact = nms_eliminates_exact(r[0], r[1], r[2], r[3], r[4], r[5], r[6], r[7], area, r[8]) ? 1 : 0;
            const NmsThetaConst th = nms_make_theta_const(r[8]);
            int fast = -1;
            if (th.fast)
                fast = nms_eliminates_fast(r[0], r[1], r[2], r[3], r[4], r[5], r[6], r[7], nms_pair_threshold(area, th.m)) ? 1 : 0;
            printf("%d %d\n", exact, fast);
        }
        fclose(f);
        return 0;
    }
    return 2;
}
