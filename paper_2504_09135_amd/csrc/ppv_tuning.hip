// Process-wide tuning and test switches.  They are read from the environment once, when the library is loaded,
// and changed afterwards only through ppv_tuning_set; no per-step call looks at the environment.
#include <cstdlib>

#include "ppv_internal.h"

namespace {

struct KnobSpec {
    const char *env;   // environment variable read at load
    int initial;       // value without it
    int lo, hi;        // accepted range
};
constexpr KnobSpec KNOBS[PPV_TUNE_COUNT] = {
    {"PPV_WAVES_PER_ROW", 0, 0, 16},   // PPV_TUNE_WAVES_PER_ROW
    {"PPV_TOPM_WAVES", 0, 0, 16},      // PPV_TUNE_TOPM_WAVES
    {"PPV_TOPM_STREAMING", 0, 0, 2},   // PPV_TUNE_TOPM_STREAMING
    {"PPV_LOOKUP", 1, 0, 1},           // PPV_TUNE_LOOKUP
    {"PPV_LOOKUP_WEAK", 0, 0, 1},      // PPV_TUNE_LOOKUP_WEAK
    {"PPV_ROW_SPLIT", 0, 0, 16},       // PPV_TUNE_ROW_SPLIT
};

struct Knobs {
    int v[PPV_TUNE_COUNT];
    Knobs() {
        for (int k = 0; k < PPV_TUNE_COUNT; k++) {
            v[k] = KNOBS[k].initial;
            if (const char *e = getenv(KNOBS[k].env)) {
                const int x = atoi(e);
                if (x >= KNOBS[k].lo && x <= KNOBS[k].hi) v[k] = x;
            }
        }
    }
};
Knobs g_knobs;   // constructed when the library is loaded

}  // namespace

int ppv_tuning(int knob) { return g_knobs.v[knob]; }

extern "C" ppv_status ppv_tuning_set(int32_t knob, int32_t value) {
    if (knob < 0 || knob >= PPV_TUNE_COUNT) return PPV_EINVAL;
    if (value < KNOBS[knob].lo || value > KNOBS[knob].hi) return PPV_ERANGE;
    g_knobs.v[knob] = value;
    return PPV_OK;
}

extern "C" ppv_status ppv_tuning_get(int32_t knob, int32_t *value) {
    if (knob < 0 || knob >= PPV_TUNE_COUNT || !value) return PPV_EINVAL;
    *value = g_knobs.v[knob];
    return PPV_OK;
}
