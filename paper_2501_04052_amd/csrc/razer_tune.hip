// Launch-shape table of the gfx950 RaZeR library and the hooks the tuner drives it with
// (include/razer_tune.h; the offline auto-tuning of Sec. 4.3 / App. E of arxiv 2501.04052).
#include "../../include/razer_tune.h"
#include "razer_kernels.hpp"

namespace razer {

namespace {

struct TunedEntry {
    int family;
    int64_t m, n, k;
    int p[4];
};
// written by `python -m paper_2501_04052_amd.tune --write` from timings on the GPU
const TunedEntry kTuned[] = {
#include "razer_tuned.inc"
    {-1, 0, 0, 0, {0, 0, 0, 0}}          // sentinel (keeps the array non-empty)
};
constexpr int kTunedCount = (int)(sizeof(kTuned) / sizeof(kTuned[0])) - 1;

struct Forced {
    bool on[RAZER_TUNE_FAMILIES] = {false, false, false, false};
    int p[RAZER_TUNE_FAMILIES][4] = {};
};
Forced& forced()
{
    static thread_local Forced f;
    return f;
}

}  // namespace

TuneShape tuned_shape(int family, int64_t m, int64_t n, int64_t k)
{
    TuneShape out{{0, 0, 0, 0}, 0};
    if (family < 0 || family >= RAZER_TUNE_FAMILIES) return out;
    const Forced& f = forced();
    if (f.on[family]) {
        for (int i = 0; i < 4; ++i) out.p[i] = f.p[family][i];
        out.source = 1;
        return out;
    }
    for (int e = 0; e < kTunedCount; ++e) {
        const TunedEntry& t = kTuned[e];
        if (t.family == family && t.m == m && t.n == n && t.k == k) {
            for (int i = 0; i < 4; ++i) out.p[i] = t.p[i];
            out.source = 2;
            return out;
        }
    }
    return out;
}

}  // namespace razer

using namespace razer;

extern "C" {

int razer_tune_force(int family, const int32_t* p)
{
    if (family == -1 && !p) {
        for (int f = 0; f < RAZER_TUNE_FAMILIES; ++f) forced().on[f] = false;
        return 0;
    }
    if (family < 0 || family >= RAZER_TUNE_FAMILIES) return 2;
    forced().on[family] = p != nullptr;
    if (p)
        for (int i = 0; i < 4; ++i) forced().p[family][i] = p[i];
    return 0;
}

int razer_tune_lookup(int family, int64_t m, int64_t rows, int64_t cols, int32_t* p)
{
    const TuneShape s = tuned_shape(family, m, rows, cols);
    if (s.source && p)
        for (int i = 0; i < 4; ++i) p[i] = s.p[i];
    return s.source;
}

int razer_tune_table_size(void) { return kTunedCount; }

}  // extern "C"
