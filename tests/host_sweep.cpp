// Host-side sweep of libsig's planning and validation logic, built with AddressSanitizer and
// UndefinedBehaviorSanitizer by tests/test_host_sanitized.py (no GPU: nothing is launched, every entry point used here is
// host only or takes a NULL context).  Any out-of-bounds access, signed overflow or other undefined arithmetic in the
// planner, the plan checks or the gradient's segment rule ends the run; the invariants below are checked on top.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <initializer_list>

#include "sig.h"

static uint64_t state = 0x9E3779B97F4A7C15ull;
static uint64_t rnd()
{
    state ^= state << 13;
    state ^= state >> 7;
    state ^= state << 17;
    return state;
}
static int64_t pick(const int64_t *v, int n) { return v[rnd() % (uint64_t)n]; }

static long checked = 0, planned = 0, failures = 0;
#define EXPECT(cond, ...) do { if (!(cond)) { ++failures; std::printf("FAILED %s: ", #cond); std::printf(__VA_ARGS__); std::printf("\n"); } } while (0)

static void one_shape(int64_t B, int64_t L, int d, int depth, int stream)
{
    ++checked;
    sig_plan_t pl;
    const int rc = sig_plan(nullptr, B, L, d, depth, stream, &pl);
    EXPECT(rc == SIG_OK || rc == SIG_ERR_INVALID || rc == SIG_ERR_TOO_LARGE, "sig_plan(%lld,%lld,%d,%d,%d) = %d", (long long)B, (long long)L, d, depth, stream, rc);
    const int segs = sig_backward_segments(nullptr, B, L, d, depth, stream);
    EXPECT(segs >= -6 && segs <= 32, "sig_backward_segments = %d", segs);
    if (rc == SIG_ERR_INVALID) EXPECT(segs == -SIG_ERR_INVALID, "arguments invalid for the forward call but not for the gradient: %d", segs);
    if (rc != SIG_OK) return;
    ++planned;
    EXPECT(pl.variant >= SIG_VARIANT_HBM_STREAMING && pl.variant <= SIG_VARIANT_LEVEL_SCAN, "variant %d", pl.variant);
    const int v = sig_plan_validate(B, L, d, depth, stream, &pl);
    EXPECT(v == SIG_OK, "the planner's own plan is refused (%d): B=%lld L=%lld d=%d depth=%d stream=%d variant=%d p=%d chunks=%d segments=%d threads=%d",
           v, (long long)B, (long long)L, d, depth, stream, pl.variant, pl.prefix_depth, pl.chunks, pl.segments, pl.threads);
    int64_t lds = 0, wgs = 0, scratch = 0;
    const int f = sig_plan_footprint(B, L, d, depth, stream, &pl, &lds, &wgs, &scratch);
    EXPECT(f == SIG_OK, "footprint %d", f);
    if (f == SIG_OK) {
        EXPECT(lds <= 64 * 1024, "LDS %lld bytes: B=%lld L=%lld d=%d depth=%d stream=%d", (long long)lds, (long long)B, (long long)L, d, depth, stream);
        EXPECT(wgs <= INT32_MAX && (wgs >= 1 || wgs == -1 || B == 0), "workgroups %lld", (long long)wgs);
        EXPECT(scratch >= 0, "scratch %lld", (long long)scratch);
    }
    if (pl.variant == SIG_VARIANT_ON_CHIP) {
        EXPECT(pl.threads >= 64 && pl.threads <= 512 && pl.threads % 64 == 0, "threads %d", pl.threads);
        EXPECT(pl.chunks >= 1 && pl.segments >= 1 && (int64_t)pl.chunks * pl.segments <= L - 1, "chunks %d segments %d for %lld increments", pl.chunks, pl.segments, (long long)(L - 1));
        EXPECT(sig_on_chip_available(d, depth, pl.prefix_depth) == 1, "no kernel for (%d,%d,%d)", d, depth, pl.prefix_depth);
        EXPECT(!stream || pl.segments == 1, "stream mode cut across workgroups");
    }
}

int main()
{
    // ---- sizes and tables
    for (int d = -1; d <= 40; ++d)
        for (int depth = -1; depth <= 70; ++depth) {
            const int64_t D = sig_size(d, depth);
            EXPECT(D >= -1, "sig_size");
            (void)sig_on_chip_available(d, depth, depth > 0 ? depth - 1 : 0);
            (void)sig_backward_available(d, depth);
        }
    for (int s = -3; s <= 12; ++s) EXPECT(sig_strerror(s) != nullptr, "sig_strerror(%d)", s);

    // ---- the planner on seeded shapes: the compiled grid (channels 2-10, depths 1-7), odd shapes beyond it, extremes
    const int64_t Bs[] = {0, 1, 2, 3, 7, 16, 64, 128, 300, 1000, 4096, 65536, 1 << 20, 5000000, (int64_t)1 << 31, (int64_t)1 << 40};
    const int64_t Ls[] = {1, 2, 3, 9, 16, 50, 100, 128, 129, 256, 257, 500, 1000, 2000, 4001, 50000, 1 << 20, (int64_t)1 << 33};
    for (int it = 0; it < 6000; ++it) {
        const int64_t B = pick(Bs, sizeof Bs / sizeof *Bs), L = pick(Ls, sizeof Ls / sizeof *Ls);
        const int d = (int)(rnd() % 11), depth = (int)(rnd() % 8), stream = (int)(rnd() % 2);
        one_shape(B, L, d, depth, stream);
    }
    for (int it = 0; it < 2000; ++it) {
        const int64_t B = (int64_t)(rnd() % 3000), L = (int64_t)(rnd() % 5000);
        const int d = (int)(rnd() % 300), depth = (int)(rnd() % 12), stream = (int)(rnd() % 3) - (int)(rnd() % 2);
        one_shape(B, L, d, depth, stream);
    }
    const int ds[] = {1, 2, 10, 255, 256, 257, 8192, 8193, 100000};
    const int depths[] = {1, 2, 8, 9, 29, 30, 31, 64};
    for (int d : ds)
        for (int depth : depths)
            for (int64_t B : {(int64_t)1, (int64_t)100, (int64_t)1 << 45})
                for (int64_t L : {(int64_t)2, (int64_t)1000, (int64_t)1 << 50})
                    for (int stream = 0; stream < 2; ++stream) one_shape(B, L, d, depth, stream);

    // ---- arbitrary plans through the checks: they may be refused, they must not misbehave
    for (int it = 0; it < 20000; ++it) {
        sig_plan_t pl;
        int32_t *f = reinterpret_cast<int32_t *>(&pl);
        for (unsigned i = 0; i < sizeof pl / sizeof(int32_t); ++i) {
            const uint64_t r = rnd();
            f[i] = (r & 7) == 0 ? (int32_t)(r >> 32) : (int32_t)((r >> 8) % 40) - 2;
        }
        pl.variant = (int32_t)(rnd() % 5);
        if (rnd() & 1) pl.threads = 64 * (int32_t)(1 + rnd() % 8);
        const int64_t B = pick(Bs, 12), L = pick(Ls, 14);
        const int d = 1 + (int)(rnd() % 10), depth = 1 + (int)(rnd() % 6), stream = (int)(rnd() % 2);
        const int v = sig_plan_validate(B, L, d, depth, stream, &pl);
        int64_t lds = 0, wgs = 0, scratch = 0;
        const int fp = sig_plan_footprint(B, L, d, depth, stream, &pl, &lds, &wgs, &scratch);
        EXPECT((v == SIG_OK) == (fp == SIG_OK), "validate %d but footprint %d", v, fp);
        if (fp == SIG_OK) EXPECT(lds <= 64 * 1024 && wgs <= INT32_MAX && scratch >= 0, "forced plan: lds %lld workgroups %lld scratch %lld", (long long)lds, (long long)wgs, (long long)scratch);
        ++checked;
    }
    EXPECT(sig_plan(nullptr, 1, 2, 2, 2, 0, nullptr) == SIG_ERR_INVALID, "NULL plan");
    EXPECT(sig_plan_validate(1, 2, 2, 2, 0, nullptr) == SIG_ERR_INVALID, "NULL plan");
    EXPECT(sig_plan_footprint(1, 2, 2, 2, 0, nullptr, nullptr, nullptr, nullptr) == SIG_ERR_INVALID, "NULL plan");

    std::printf("host sweep: %ld cases, %ld planned, %ld failures\n", checked, planned, failures);
    if (failures == 0) std::printf("host sweep ok\n");
    return failures == 0 ? 0 : 1;
}
