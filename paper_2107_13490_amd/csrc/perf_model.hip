// The paper's analytical performance model (Sec. 4.1 "Performance Model"): per-step training cost
// of a set of layers weighted by word length and sparsity, the bounds on the PushDown / PushUp
// overhead, model size, memory, and the speed-up quotient.  Host functions only: they turn the
// per-layer <WL>, sparsity, lookback and resolution that the kernels produce into the paper's
// figures of merit, for side-by-side context with measured times.
#include <cmath>

#include "adapt_fxp.h"

extern "C" double adapt_perf_pushdown_ops(int resolution, double numel)
{
    return 2.0 * std::log2(32.0 - 8.0) * (double)resolution * 3.0 * numel;
}

extern "C" double adapt_perf_pushup_ops(int lookback, double numel) { return ((double)lookback + 1.0) * numel + 1.0; }

extern "C" double adapt_perf_step_cost(const adapt_perf_layer *layers, int count, int accs)
{
    if (!layers || count < 0 || accs < 1) return NAN;
    double c = 0.0;
    for (int l = 0; l < count; ++l) c += layers[l].ops * (layers[l].sp * (double)layers[l].wl + 32.0 / (double)accs);
    return c;
}

extern "C" double adapt_perf_step_overhead(const adapt_perf_layer *layers, int count, int accs)
{
    if (!layers || count < 0 || accs < 1) return NAN;
    double c = 0.0;
    for (int l = 0; l < count; ++l) {
        if (layers[l].lookback < 1) return NAN;
        const double pd = adapt_perf_pushdown_ops(layers[l].resolution, layers[l].numel);
        const double pu = adapt_perf_pushup_ops(layers[l].lookback, layers[l].numel);
        c += 32.0 * (layers[l].sp * pd + pu) / ((double)accs * (double)layers[l].lookback);
    }
    return c;
}

extern "C" double adapt_perf_model_size(const adapt_perf_layer *layers, int count)
{
    if (!layers || count < 0) return NAN;
    double c = 0.0;
    for (int l = 0; l < count; ++l) c += layers[l].sp * (double)layers[l].wl;
    return c;
}

extern "C" double adapt_perf_step_memory(const adapt_perf_layer *layers, int count)
{
    if (!layers || count < 0) return NAN;
    double c = 0.0;
    for (int l = 0; l < count; ++l) c += layers[l].sp * (double)layers[l].wl + 32.0;
    return c;
}

extern "C" double adapt_perf_speedup(double bs_other, double costs_other, double bs_ours, double costs_ours)
{
    return bs_other * costs_other / (bs_ours * costs_ours);
}
