// Phase trace of a kernel, for builds with -DLORA_TRACE only (a development aid, never part of the shipped library:
// it allocates, synchronises and reads the environment, which the library proper never does).
#pragma once
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

namespace lora {
// ---- optional phase trace: builds with -DLORA_TRACE only (a development aid) -------------------------------
// Thread 0 of every workgroup stamps the constant 100 MHz clock into trace[blockIdx.x * 8 + slot]; with the
// environment variable LORA_TRACE set to a kernel's name, that kernel's 30th launch prints the stamps in
// microseconds relative to the earliest one (the launches are synchronous then).
#define LORA_TS(buf, i)                                                                     \
    do {                                                                                    \
        if ((buf) != nullptr && threadIdx.x == 0) (buf)[blockIdx.x * 8 + (i)] = wall_clock64(); \
    } while (0)
// the same from the first thread of wave `w` (how far apart the waves of a workgroup finish a phase)
#define LORA_TS_WAVE(buf, i, w)                                                                              \
    do {                                                                                                     \
        if ((buf) != nullptr && (int)threadIdx.x == (w) * 64) (buf)[blockIdx.x * 8 + (i)] = wall_clock64(); \
    } while (0)
template <typename Launch>
inline hipError_t trace_launch(const char *name, long grid, Launch launch) {
    const char *want = getenv("LORA_TRACE");
    if (want == nullptr || strcmp(want, name) != 0) return launch(nullptr);
    constexpr long kMaxWgs = 8192;
    static long long *dbuf = nullptr;
    static int calls = 0;
    if (dbuf == nullptr && hipMalloc(&dbuf, 8 * 8 * kMaxWgs) != hipSuccess) return hipErrorOutOfMemory;
    (void)hipMemset(dbuf, 0, 8 * 8 * kMaxWgs);
    (void)hipDeviceSynchronize();
    hipError_t e = grid <= kMaxWgs ? launch(dbuf) : launch(nullptr);
    (void)hipDeviceSynchronize();
    if (++calls == 30 && grid <= kMaxWgs) {
        static long long h[8 * kMaxWgs];
        (void)hipMemcpy(h, dbuf, sizeof(long long) * 8 * grid, hipMemcpyDeviceToHost);
        long long t0 = -1;
        for (long g = 0; g < grid; ++g)
            if (h[g * 8] && (t0 < 0 || h[g * 8] < t0)) t0 = h[g * 8];
        const long stride = getenv("LORA_TRACE_ALL") ? 1 : (grid > 48 ? grid / 24 : 1);  // a sample of the workgroups, or all
        for (long g = 0; g < grid; g += stride) {
            if (!h[g * 8]) continue;
            printf("trace %s wg %ld:", name, g);
            for (int i = 0; i < 8; ++i) printf(" %6.2f", h[g * 8 + i] ? (h[g * 8 + i] - t0) * 0.01 : -1.0);
            printf("\n");
        }
        fflush(stdout);
    }
    return e;
}

}  // namespace lora
