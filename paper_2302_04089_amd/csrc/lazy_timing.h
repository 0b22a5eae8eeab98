// Optional phase timing of the single-column greedy loop (prune_lazy.hip).  A build with -DZIPLM_LAZY_TIMING reads
// the 100 MHz wall clock at the phase boundaries of workgroup 0 and prints the sums to stderr after every launch
// (which then waits for the stream); the regular build compiles every macro below to nothing.
#pragma once

#ifndef ZIPLM_LAZY_TIMING

#define ZIPLM_LAZY_TIMING_FIELD
#define ZIPLM_LAZY_TIMING_LOCALS
#define TICK(slot) do { } while (0)
#define ZIPLM_LAZY_TIMING_LOCAL_DONE do { } while (0)
#define ZIPLM_LAZY_TIMING_OWN_SLOT do { } while (0)
#define ZIPLM_LAZY_TIMING_EXCHANGE_DONE do { } while (0)
#define ZIPLM_LAZY_TIMING_PAYLOAD_SEEN(word) do { } while (0)
#define ZIPLM_LAZY_TIMING_WRITE_BACK do { } while (0)
#define ZIPLM_LAZY_TIMING_TAKE(state, carver) do { } while (0)
#define ZIPLM_LAZY_TIMING_REPORT(state, nb, n_remove, stream) do { } while (0)

#else

#include <stdio.h>

// [8] accumulated ticks per phase (workgroup 0), [1024] per-workgroup local ticks, [2] payload-visible counters
#define ZIPLM_LAZY_TIMING_FIELD unsigned long long *timing;
#define ZIPLM_LAZY_TIMING_LOCALS                                           \
    unsigned long long tacc[8] = {0, 0, 0, 0, 0, 0, 0, 0};                 \
    unsigned long long tlast = wall_clock64();                             \
    unsigned long long tlocal = 0, texch = wall_clock64();
#define TICK(slot) do { if (b == 0 && tid == 0) { const unsigned long long now_ = wall_clock64(); tacc[slot] += now_ - tlast; tlast = now_; } } while (0)
// time from "exchange done" to "slot of the next step published" (thread 0 of every workgroup)
#define ZIPLM_LAZY_TIMING_LOCAL_DONE do { tlocal += wall_clock64() - texch; } while (0)
// own slot seen again: store -> load round trip
#define ZIPLM_LAZY_TIMING_OWN_SLOT do { if (b == 0 && tid == 0) tacc[7] += wall_clock64() - tlast; } while (0)
#define ZIPLM_LAZY_TIMING_EXCHANGE_DONE do { if (tid == 0) texch = wall_clock64(); } while (0)
// was the winner's payload there at the first look?
#define ZIPLM_LAZY_TIMING_PAYLOAD_SEEN(word) do {                                                   \
        if (b == 1 && tid3 == 64 && owner != b) {                                                   \
            S.timing[8 + 1024] += 1;                                                                \
            S.timing[8 + 1025] += ((unsigned)((word) & 0xffffffffu) == tag) ? 1 : 0;                \
        }                                                                                           \
    } while (0)
#define ZIPLM_LAZY_TIMING_WRITE_BACK do {                                           \
        if (b == 0 && tid == 0) for (int q = 0; q < 8; ++q) S.timing[q] = tacc[q];  \
        if (tid == 0) S.timing[8 + b] = tlocal;                                     \
    } while (0)
#define ZIPLM_LAZY_TIMING_TAKE(state, carver) do { (state).timing = (carver).take<unsigned long long>(8 + 1024 + 8); } while (0)
#define ZIPLM_LAZY_TIMING_REPORT(state, nb, n_remove, stream) ziplm_lazy_timing_report((state).timing, (nb), (n_remove), (stream))

static inline void ziplm_lazy_timing_report(const unsigned long long *timing, int nb, int n_remove, hipStream_t st) {
    const int steps = n_remove > 0 ? n_remove : 1;
    unsigned long long tm[8], loc[1024], pr[2];
    hipStreamSynchronize(st);
    hipMemcpy(tm, timing, sizeof(tm), hipMemcpyDeviceToHost);
    hipMemcpy(loc, timing + 8, sizeof(unsigned long long) * nb, hipMemcpyDeviceToHost);
    hipMemcpy(pr, timing + 8 + 1024, sizeof(pr), hipMemcpyDeviceToHost);
    const char *names[8] = {"snapshot+loop top", "candidate+publish", "exchange+argmin", "payload+gather", "row slice + Eq.3",
                            "flush barrier", "flush update", "(own slot round trip)"};
    for (int q = 0; q < 8; ++q)
        fprintf(stderr, "[lazy timing] %-20s %9.3f ms total  %7.3f us/step\n", names[q], tm[q] * 1e-5, tm[q] * 1e-2 / steps);
    double mn = 1e30, mx = 0, sum = 0;
    int imx = 0;
    for (int q = 0; q < nb; ++q) {
        const double v = loc[q] * 1e-2 / steps;
        sum += v;
        if (v < mn) mn = v;
        if (v > mx) { mx = v; imx = q; }
    }
    fprintf(stderr, "[lazy timing] local us/step (exchange done -> slot published): min %.3f avg %.3f max %.3f (block %d)\n", mn, sum / nb, mx, imx);
    if (pr[0])
        fprintf(stderr, "[lazy timing] winner's payload already visible at the first read of step 3: %.1f%% of %llu steps (workgroup 1)\n",
                100.0 * pr[1] / pr[0], pr[0]);
    double x[8] = {0};
    int c[8] = {0};
    for (int q = 0; q < nb; ++q) { x[q & 7] += loc[q] * 1e-2 / steps; c[q & 7]++; }
    fprintf(stderr, "[lazy timing] local us/step by workgroup index mod 8:");
    for (int q = 0; q < 8; ++q) fprintf(stderr, " %.3f", x[q] / (c[q] ? c[q] : 1));
    fprintf(stderr, "\n[lazy timing] local us/step by workgroup index / 32:");
    for (int g = 0; g < 8; ++g) {
        double a = 0;
        int n = 0;
        for (int q = 32 * g; q < 32 * g + 32 && q < nb; ++q) { a += loc[q] * 1e-2 / steps; ++n; }
        fprintf(stderr, " %.3f", n ? a / n : 0.0);
    }
    fprintf(stderr, "\n");
}

#endif
