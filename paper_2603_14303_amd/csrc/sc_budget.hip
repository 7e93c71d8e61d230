// sc_gsc_merge_budget: sc_gsc_merge with the similarity threshold chosen for a target cache size.
//
// The paper reports its results at cache budgets (Sec. 3.1: 20 / 35 / 50 % of the entries kept) but does
// not say how a budget becomes the threshold tau of Alg. 1.  The number of rows N'(tau) grows with tau
// (a higher bar merges less), so the largest tau that still meets the budget is found by bisection.
// Every probe is the clustering half of sc_gsc_merge (counts only); the threshold lives in device memory.
// A probe ends in the scan kernel, whose workgroups (one per sequence and head) add up their row counts;
// the last of them to arrive moves the bracket and writes the next threshold (where a probe is a complete
// merge, outside the bf16 / d = 128 path, a small kernel after it does that from the merged lengths).  The
// whole search is a fixed sequence of launches on the caller's stream with no host synchronisation.  The
// last launch runs at the threshold found and leaves its merged cache in the outputs.
#include "sc_device.h"
#include "sc_gsc_params.h"
#include "sc_host.h"

namespace sc {

size_t gsc_budget_state_bytes() { return align_up(sizeof(BudgetState), 256); }

__global__ void budget_init_kernel(BudgetState *st, float lo, float hi, long long budget_rows, int iterations, float *tau_out,
                                   long long *rows_out) {
    st->lo = lo;
    st->hi = hi;
    st->step = 0;
    st->rows_lo = -1;
    st->tau = (iterations > 0) ? 0.5f * (lo + hi) : lo;   // no probe: the final launch runs at tau_lo
    st->budget_rows = budget_rows;
    st->iterations = iterations;
    st->tau_out = tau_out;
    st->rows_out = rows_out;
    st->arrived = 0u;
    st->bad = 0;
    st->total = 0;
}

// after a complete merge at st->tau: total rows from the merged lengths (any overflowed head counts as over
// budget), then the same step as after a counting probe
__global__ __launch_bounds__(256) void budget_update_kernel(BudgetState *st, const int32_t *comp_lens, int n_bh) {
    __shared__ long long s_sum[256];
    __shared__ int s_bad[256];
    long long sum = 0;
    int bad = 0;
    for (int i = threadIdx.x; i < n_bh; i += 256) {
        const int v = comp_lens[i];
        if (v < 0) bad = 1; else sum += v;
    }
    s_sum[threadIdx.x] = sum;
    s_bad[threadIdx.x] = bad;
    __syncthreads();
    if (threadIdx.x != 0) return;
    for (int i = 1; i < 256; ++i) { sum += s_sum[i]; bad |= s_bad[i]; }
    budget_bracket_step(st, sum, bad != 0);
}

hipError_t launch_gsc_budget(GscMergeArgs a, long long budget_rows, float tau_lo, float tau_hi, int iterations,
                             float *tau_out, long long *rows_out, void *state, hipStream_t stream) {
    BudgetState *st = reinterpret_cast<BudgetState *>(state);
    hipLaunchKernelGGL(budget_init_kernel, dim3(1), dim3(1), 0, stream, st, tau_lo, tau_hi, budget_rows, iterations, tau_out, rows_out);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    a.tau_dev = &st->tau;
    const bool counting = gsc_merge_takes_fast_path(a);
    for (int it = 0; it <= iterations; ++it) {     // `iterations` probes, then the launch at the result
        // a probe only needs the row counts: clustering without reading the values, without the merge and
        // without writing rows, and its scan kernel moves the bracket itself (where the fast path runs;
        // elsewhere a probe is a full merge followed by the update kernel, like the final launch)
        const bool probe = it < iterations;
        a.count_only = probe;
        a.budget_state = (probe && counting) ? state : nullptr;
        e = launch_gsc_merge(a, stream);
        if (e != hipSuccess) return e;
        if (!(probe && counting)) {
            hipLaunchKernelGGL(budget_update_kernel, dim3(1), dim3(256), 0, stream, st, a.comp_lens, a.B * a.Hkv);
            e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
    }
    return hipSuccess;
}

}  // namespace sc
