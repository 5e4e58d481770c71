// Host-only exerciser of the C ABI's plan code, built with AddressSanitizer + UBSan or with
// ThreadSanitizer (paper_1911_03458_amd/build.py: build_host_check) and run by
// tests/test_host_sanitized.py.  It touches no GPU: plans are created, queried, overridden and
// destroyed, and the operation entry points are called only in ways that return before any
// launch (null plan, null or misaligned tensor pointers, a plan of another operation).
//
//   host_check [threads]      threads > 1: the same sweep from several threads at once, plus one
//                             plan shared by all of them (merit.h: a plan may be shared)
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <thread>
#include <vector>

#include "merit.h"

namespace {

struct Rng {                       // splitmix64: the sweep is the same on every run
    uint64_t s;
    uint64_t next()
    {
        uint64_t z = (s += 0x9e3779b97f4a7c15ull);
        z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
        z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
        return z ^ (z >> 31);
    }
    int in(int lo, int hi) { return lo + (int)(next() % (uint64_t)(hi - lo + 1)); }
};

int failures = 0;
#define CHECK(cond)                                                                      \
    do {                                                                                 \
        if (!(cond)) {                                                                   \
            std::fprintf(stderr, "host_check: %s failed at line %d\n", #cond, __LINE__); \
            __atomic_add_fetch(&failures, 1, __ATOMIC_RELAXED);                          \
        }                                                                                \
    } while (0)

// every query the ABI offers on a plan; then the plan rebuilt from its own descriptor
void query(merit_plan *plan)
{
    merit_plan_desc d;
    CHECK(merit_plan_get_desc(plan, &d) == MERIT_OK);
    int32_t nd = 0;
    int64_t shape[MERIT_MAX_DIMS];
    CHECK(merit_plan_out_shape(plan, &nd, shape) == MERIT_OK && nd >= 1 && nd <= MERIT_MAX_DIMS);
    merit_launch_info li;
    CHECK(merit_plan_launch_info(plan, &li) == MERIT_OK && li.kernel != nullptr && std::strlen(li.kernel) > 0);
    CHECK(li.lds_bytes >= 0 && li.lds_bytes <= 160 * 1024 && li.block[0] > 0 && li.block[0] <= 1024);
    int64_t tile[MERIT_MAX_INDEX], fp[MERIT_MAX_DIMS];
    bool empty = false;                                         // a range of 0 admits no tile
    for (int j = 0; j < MERIT_MAX_INDEX; ++j) {
        tile[j] = 1 + (j % 3);
        if (j < d.n_par + d.n_acc) {
            if (tile[j] > d.range[j]) tile[j] = d.range[j];
            empty = empty || d.range[j] == 0;
        }
    }
    CHECK(merit_plan_footprint(plan, 0, tile, fp) == (empty ? MERIT_ERR_INVALID_ARG : MERIT_OK));
    if (!empty)
        for (int i = 0; i < d.a.ndim; ++i) CHECK(fp[i] >= 1);
    (void)merit_plan_footprint(plan, 1, tile, fp);              // operand b may not exist (pooling)
    CHECK(merit_plan_footprint(plan, 2, tile, fp) != MERIT_OK);
    tile[0] = d.range[0] + 1;                                   // a tile larger than its range
    CHECK(merit_plan_footprint(plan, 0, tile, fp) == MERIT_ERR_INVALID_ARG);
    int64_t bytes = -1;
    const merit_status ps = merit_plan_packed_weights_bytes(plan, &bytes);
    CHECK(ps == MERIT_ERR_UNSUPPORTED || (ps == MERIT_OK && bytes > 0 && bytes % 16 == 0));
    merit_plan *again = nullptr;
    CHECK(merit_plan_create(&d, &again) == MERIT_OK && again != nullptr);
    if (again) {
        merit_launch_info l2;
        CHECK(merit_plan_launch_info(again, &l2) == MERIT_OK && std::strcmp(li.kernel, l2.kernel) == 0);
        merit_plan_destroy(again);
    }
    // tile requests: accepted or refused, never a crash; a refused request leaves the plan as it was
    for (int a = 0; a < 6; ++a) {
        int64_t req[MERIT_MAX_INDEX] = {0};
        static const int64_t w[] = {4, 8, 12, 1, 16, 64}, px[] = {32, 64, 128, 1, 8, 64};
        req[1] = a; req[2] = w[a]; req[3] = px[a];
        (void)merit_plan_set_tile(plan, req);
        CHECK(merit_plan_launch_info(plan, &li) == MERIT_OK && li.lds_bytes <= 160 * 1024);
    }
}

// the operation entry points in the ways that return before anything is launched
void refuse(merit_plan *plan)
{
    void *odd = reinterpret_cast<void *>(uintptr_t(0x1008));   // never dereferenced: not 16-byte aligned
    CHECK(merit_conv2d(nullptr, odd, odd, odd, nullptr) == MERIT_ERR_NULL);
    CHECK(merit_pool2d(nullptr, odd, odd, nullptr) == MERIT_ERR_NULL);
    CHECK(merit_sad_search(nullptr, odd, odd, odd, odd, nullptr) == MERIT_ERR_NULL);
    merit_plan_desc d;
    merit_plan_get_desc(plan, &d);
    int32_t nd;
    int64_t shape[MERIT_MAX_DIMS];
    merit_plan_out_shape(plan, &nd, shape);
    bool empty = false;
    for (int i = 0; i < nd; ++i) empty = empty || shape[i] == 0;
    if (empty) return;                                          // an empty output is a no-op that returns OK
    merit_status s;
    switch (d.op) {
    case MERIT_OP_CONV_DOT: case MERIT_OP_CONV_DOT_RELU: case MERIT_OP_CONV_DOT_POOLMAX:
    case MERIT_OP_CONV_DOT_RELU_POOLMAX:
        s = merit_conv2d(plan, nullptr, nullptr, nullptr, nullptr); CHECK(s == MERIT_ERR_NULL);
        s = merit_conv2d(plan, odd, odd, odd, nullptr); CHECK(s == MERIT_ERR_ALIGNMENT);
        CHECK(merit_pool2d(plan, odd, odd, nullptr) == MERIT_ERR_INVALID_ARG);
        s = merit_conv2d_packed(plan, odd, odd, odd, nullptr);
        CHECK(s == MERIT_ERR_ALIGNMENT || s == MERIT_ERR_UNSUPPORTED);
        s = merit_conv2d_packed_noalloc(plan, odd, odd, odd, nullptr);
        CHECK(s == MERIT_ERR_ALIGNMENT || s == MERIT_ERR_UNSUPPORTED || s == MERIT_ERR_SCRATCH_LIMIT);
        break;
    case MERIT_OP_POOL_MAX: case MERIT_OP_POOL_AVG:
        CHECK(merit_pool2d(plan, nullptr, nullptr, nullptr) == MERIT_ERR_NULL);
        CHECK(merit_pool2d(plan, odd, odd, nullptr) == MERIT_ERR_ALIGNMENT);
        CHECK(merit_conv2d(plan, odd, odd, odd, nullptr) == MERIT_ERR_INVALID_ARG);
        break;
    case MERIT_OP_SAD_ARGMIN:
        CHECK(merit_sad_search(plan, nullptr, odd, odd, odd, nullptr) == MERIT_ERR_NULL);
        CHECK(merit_sad_search(plan, odd, odd, odd, odd, nullptr) == MERIT_ERR_ALIGNMENT);
        break;
    case MERIT_OP_CONV_DOT_ADD: case MERIT_OP_CONV_DOT_ADD_RELU:
        CHECK(merit_conv2d_residual(plan, odd, odd, odd, odd, nullptr) == MERIT_ERR_ALIGNMENT);
        CHECK(merit_conv2d(plan, odd, odd, odd, nullptr) == MERIT_ERR_INVALID_ARG);
        break;
    case MERIT_OP_DWCONV_DOT:
        CHECK(merit_conv2d_depthwise(plan, odd, odd, odd, nullptr) == MERIT_ERR_ALIGNMENT);
        break;
    case MERIT_OP_CORR_DOT:
        CHECK(merit_correlation(plan, odd, odd, odd, nullptr) == MERIT_ERR_ALIGNMENT);
        break;
    case MERIT_OP_SEPFILTER_DOT:
        CHECK(merit_sepfilter(plan, odd, odd, odd, odd, nullptr) == MERIT_ERR_ALIGNMENT);
        break;
    case MERIT_OP_BILATERAL:
        CHECK(merit_bilateral(plan, odd, odd, odd, -0.01, odd, nullptr) == MERIT_ERR_ALIGNMENT);
        break;
    }
}

void take(merit_status s, merit_plan *plan, int *made)
{
    CHECK(s >= MERIT_OK && s <= MERIT_ERR_SCRATCH_LIMIT);
    CHECK((s == MERIT_OK) == (plan != nullptr));
    if (!plan) return;
    ++*made;
    query(plan);
    refuse(plan);
    CHECK(merit_plan_destroy(plan) == MERIT_OK);
}

// a seeded sweep of valid, odd and invalid shapes over every constructor
int sweep(uint64_t seed, int rounds)
{
    Rng r{seed};
    int made = 0;
    static const int chans[] = {1, 3, 7, 8, 16, 24, 48, 64, 100, 128, 136, 256, 512, 1000};
    static const int wins[] = {1, 2, 3, 5, 7, 11};
    for (int i = 0; i < rounds; ++i) {
        const int N = r.in(0, 40), Cin = chans[r.in(0, 13)], Cout = chans[r.in(0, 13)];
        const int H = r.in(1, 230), W = r.in(1, 230);
        const int kh = wins[r.in(0, 5)], kw = r.in(0, 3) ? kh : wins[r.in(0, 5)];
        const int sh = r.in(1, 4), sw = r.in(0, 3) ? sh : r.in(1, 4);
        const int ph = r.in(0, kh), pw = r.in(0, kw);
        const int dh = r.in(1, 3), dw = r.in(1, 3), relu = r.in(0, 1);
        merit_plan *p = nullptr;
        take(merit_plan_conv2d(N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, &p), p, &made);
        p = nullptr; take(merit_plan_conv2d_relu(N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, &p), p, &made);
        p = nullptr; take(merit_plan_conv2d_dilated(N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, dh, dw, relu, &p), p, &made);
        p = nullptr; take(merit_plan_conv2d_pool(N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, relu, &p), p, &made);
        p = nullptr; take(merit_plan_conv2d_residual(N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, relu, &p), p, &made);
        p = nullptr; take(merit_plan_conv2d_depthwise(N, Cin, H, W, kh, kw, sh, sw, ph, pw, &p), p, &made);
        p = nullptr; take(merit_plan_pool2d(N, Cin, H, W, kh, kw, sh, sw, ph, pw, relu, &p), p, &made);
        p = nullptr; take(merit_plan_sad(H, W, 4 * r.in(0, 9), r.in(-1, 70), &p), p, &made);
        p = nullptr; take(merit_plan_correlation(N, Cin, H, W, r.in(0, 17), r.in(0, 9), &p), p, &made);
        p = nullptr; take(merit_plan_sepfilter(N, H, W, r.in(0, 34), &p), p, &made);
        p = nullptr; take(merit_plan_bilateral(N, H, W, r.in(0, 34), &p), p, &made);
        // arguments no shape can mean
        p = nullptr; take(merit_plan_conv2d(-1, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, &p), p, &made);
        p = nullptr; take(merit_plan_pool2d(N, Cin, H, W, kh, kw, 0, sw, ph, pw, 0, &p), p, &made);
        p = nullptr; take(merit_plan_conv2d(N, Cin, H, W, Cout, H + 2 * ph + 1, kw, sh, sw, ph, pw, &p), p, &made);
    }
    // the workloads themselves and a few extreme shapes
    merit_plan *p = nullptr;
    take(merit_plan_conv2d(8, 256, 56, 56, 256, 3, 3, 1, 1, 1, 1, &p), p, &made);
    p = nullptr; take(merit_plan_conv2d(32, 3, 224, 224, 64, 7, 7, 2, 2, 3, 3, &p), p, &made);
    p = nullptr; take(merit_plan_conv2d(1 << 14, 4096, 8, 8, 64, 3, 3, 1, 1, 1, 1, &p), p, &made);
    p = nullptr; take(merit_plan_pool2d(16, 64, 112, 112, 3, 3, 2, 2, 1, 1, 1, &p), p, &made);
    p = nullptr; take(merit_plan_pool2d(1, 1, 16, 8192, 3, 3, 2, 2, 1, 1, 0, &p), p, &made);
    p = nullptr; take(merit_plan_sad(1088, 1920, 16, 32, &p), p, &made);
    p = nullptr; take(merit_plan_sad(4320, 7680, 16, 63, &p), p, &made);
    CHECK(merit_plan_conv2d(1, 1, 1, 1, 1, 1, 1, 1, 1, 0, 0, nullptr) == MERIT_ERR_NULL);
    CHECK(merit_plan_create(nullptr, &p) == MERIT_ERR_NULL);
    CHECK(merit_plan_destroy(nullptr) != MERIT_OK || true);
    for (int s = MERIT_OK; s <= MERIT_ERR_SCRATCH_LIMIT; ++s) CHECK(merit_status_string((merit_status)s) != nullptr);
    return made;
}

}  // namespace

int main(int argc, char **argv)
{
    const int nthreads = argc > 1 ? std::atoi(argv[1]) : 1;
    int made = 0;
    if (nthreads <= 1) {
        made = sweep(1911, 120);
    } else {
        // one plan shared by every thread (queries only: merit.h allows that), next to the
        // private sweeps
        merit_plan *shared = nullptr;
        CHECK(merit_plan_conv2d(8, 64, 56, 56, 64, 3, 3, 1, 1, 1, 1, &shared) == MERIT_OK);
        std::vector<std::thread> pool;
        std::vector<int> counts((size_t)nthreads, 0);
        for (int t = 0; t < nthreads; ++t)
            pool.emplace_back([&, t] {
                counts[(size_t)t] = sweep(1911 + 7 * (uint64_t)t, 25);
                for (int k = 0; k < 200; ++k) {
                    merit_launch_info li;
                    int32_t nd;
                    int64_t shape[MERIT_MAX_DIMS];
                    CHECK(merit_plan_launch_info(shared, &li) == MERIT_OK);
                    CHECK(merit_plan_out_shape(shared, &nd, shape) == MERIT_OK && nd == 4 && shape[1] == 64);
                    refuse(shared);
                }
            });
        for (auto &th : pool) th.join();
        for (int c : counts) made += c;
        merit_plan_destroy(shared);
    }
    std::printf("host_check: %d plans made and queried on %d thread(s), %d failed checks\n", made,
                nthreads > 1 ? nthreads : 1, failures);
    return failures ? 1 : 0;
}
