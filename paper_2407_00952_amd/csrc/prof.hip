// Event-based timing of kernel launches (see prof.h).  Host code only.
#include "prof.h"
#include "common.h"
#include <vector>

namespace {
struct Prof {
    unsigned mask = 0;
    std::vector<hipEvent_t> ev;      // pairs: start, stop
    std::vector<int> kind;           // per pair
    std::vector<double> work;        // per pair
    size_t used = 0;                 // pairs recorded
} g;
constexpr size_t kMaxPairs = 16384;
}  // namespace

int prof_enable(unsigned mask)
{
    if (mask && g.ev.empty()) {
        g.ev.resize(2 * kMaxPairs);
        for (auto &e : g.ev)
            if (hipEventCreate(&e) != hipSuccess) { g.ev.clear(); return SL_EHIP; }
        g.kind.resize(kMaxPairs);
        g.work.resize(kMaxPairs);
    }
    g.mask = mask;
    g.used = 0;
    return SL_OK;
}

bool prof_begin(int kind, hipStream_t st)
{
    if (!((g.mask >> kind) & 1u) || g.used >= kMaxPairs) return false;
    (void)hipEventRecord(g.ev[2 * g.used], st);
    return true;
}

void prof_end(bool recording, int kind, double work, hipStream_t st)
{
    if (!recording) return;
    (void)hipEventRecord(g.ev[2 * g.used + 1], st);
    g.kind[g.used] = kind;
    g.work[g.used] = work;
    ++g.used;
}

int prof_read(int kind, double *ms, double *work, int *launches)
{
    double tot = 0.0, w = 0.0;
    int n = 0;
    for (size_t i = 0; i < g.used; ++i) {
        if (g.kind[i] != kind) continue;
        float t = 0.f;
        if (hipEventSynchronize(g.ev[2 * i + 1]) != hipSuccess) return SL_EHIP;
        if (hipEventElapsedTime(&t, g.ev[2 * i], g.ev[2 * i + 1]) != hipSuccess) return SL_EHIP;
        tot += t;
        w += g.work[i];
        ++n;
    }
    if (ms) *ms = tot;
    if (work) *work = w;
    if (launches) *launches = n;
    return SL_OK;
}
