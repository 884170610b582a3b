// Event-based timing of kernel launches (see prof.h).  Host code only.
#include "prof.h"
#include "common.h"
#include <vector>

// clock stamps of the recorded GEMM launches: [pair][4] = shader clock at start, reference clock at start,
// shader clock at end, reference clock at end (written by block 0 of the 4-wave GEMM kernel)
static __device__ unsigned long long clock_words[16384 * 4];

namespace {
struct Prof {
    unsigned mask = 0;
    std::vector<hipEvent_t> ev;      // pairs: start, stop
    std::vector<int> kind;           // per pair
    std::vector<double> work;        // per pair
    size_t used = 0;                 // pairs recorded
    unsigned long long *clk = nullptr;   // device address of clock_words on the device profiling was enabled on
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
    if (mask && !g.clk) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(clock_words)) != hipSuccess) return SL_EHIP;
        g.clk = (unsigned long long *)p;
    }
    if (mask && hipMemset(g.clk, 0, sizeof(unsigned long long) * 4 * kMaxPairs) != hipSuccess) return SL_EHIP;
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

unsigned long long *prof_clock_words(bool recording)
{
    return (recording && g.clk) ? g.clk + 4 * g.used : nullptr;
}

int prof_read_clock(double *mhz, int *samples)
{
    double shader = 0.0, ref = 0.0;
    int n = 0;
    if (g.clk && g.used) {
        if (hipDeviceSynchronize() != hipSuccess) return SL_EHIP;
        std::vector<unsigned long long> h(4 * g.used);
        if (hipMemcpy(h.data(), g.clk, sizeof(unsigned long long) * h.size(), hipMemcpyDeviceToHost) != hipSuccess)
            return SL_EHIP;
        for (size_t i = 0; i < g.used; ++i) {
            const unsigned long long *w = &h[4 * i];
            if (g.kind[i] != PK_GEMM || w[3] <= w[1] || w[2] <= w[0]) continue;
            shader += (double)(w[2] - w[0]);
            ref += (double)(w[3] - w[1]);
            ++n;
        }
    }
    if (mhz) *mhz = ref > 0.0 ? shader / ref * 100.0 : 0.0;     // the reference counter runs at 100 MHz
    if (samples) *samples = n;
    return SL_OK;
}
