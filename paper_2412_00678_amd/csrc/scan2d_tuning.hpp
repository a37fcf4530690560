// Tuning overrides of the dispatcher.  They start from the environment, read ONCE per process (first use),
// and can afterwards only be changed through scan2d_debug_force_variant (a test hook): the entry points
// themselves never call getenv.
//   SCAN2D_FWD_VARIANT = LG,K,NW,WAVES[,RPB]     force a variant of the plain forward kernel
//   SCAN2D_FWD_SHARED  = LG,K,NW,WAVES,RPB[,SKEW] force a variant of the shared-producer forward kernel (SKEW = 1: its
//                        skewed-row tilings; "0" alone = never use that form)
//   SCAN2D_BWD_VARIANT = LG,K[,WAVES[,GS]]       force a variant of the banded backward
#pragma once

#include <atomic>

namespace scan2d {

enum { kTuneFwd = 0, kTuneShared = 1, kTuneBwd = 2, kTuneKinds = 3, kTuneMaxValues = 6 };

struct TuneSlot {
    std::atomic<int> n{0};                       // number of values given (0 = no override)
    std::atomic<int> v[kTuneMaxValues];
};

// Snapshot of one override (plain ints, taken once per call).
struct TuneValues {
    int n = 0;
    int v[kTuneMaxValues] = {0, 0, 0, 0, 0, 0};
};

TuneValues tune_get(int kind);                   // reads the environment on first use
void tune_set(int kind, const int* values, int n);

}  // namespace scan2d
