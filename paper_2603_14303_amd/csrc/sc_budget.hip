// sc_gsc_merge_budget: sc_gsc_merge with the similarity threshold chosen for a target cache size.
//
// The paper reports its results at cache budgets (Sec. 3.1: 20 / 35 / 50 % of the entries kept) but does
// not say how a budget becomes the threshold tau of Alg. 1.  The number of rows N'(tau) grows with tau
// (a higher bar merges less), so the largest tau that still meets the budget is found by bisection.
// Every probe is the clustering half of sc_gsc_merge (counts only); the threshold lives in device memory, a one-thread kernel
// between two probes reads the merged lengths of the last one and moves the bracket, so the whole
// search is a fixed sequence of launches on the caller's stream with no host synchronisation.  The
// last launch runs at the threshold found and leaves its merged cache in the outputs.
#include "sc_device.h"
#include "sc_host.h"

namespace sc {

struct BudgetState {
    float tau;            // threshold of the next sc_gsc_merge launch
    float lo, hi;         // bracket: lo is assumed to meet the budget, hi not to
    int step;
    long long rows_lo;    // rows at lo (-1 until lo itself has been probed)
};

size_t gsc_budget_state_bytes() { return align_up(sizeof(BudgetState), 256); }

__global__ void budget_init_kernel(BudgetState *st, float lo, float hi) {
    st->lo = lo;
    st->hi = hi;
    st->step = 0;
    st->rows_lo = -1;
    st->tau = 0.5f * (lo + hi);
}

// after a probe at st->tau: total rows (any overflowed head counts as over budget), move the bracket,
// choose the next threshold: another midpoint, or lo itself for the final launch
__global__ __launch_bounds__(256) void budget_update_kernel(BudgetState *st, const int32_t *comp_lens, int n_bh,
                                                           long long budget_rows, int iterations, float *tau_out,
                                                           long long *rows_out) {
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
    const int step = st->step;
    if (step < iterations) {
        const bool fits = !bad && sum <= budget_rows;
        if (fits) { st->lo = st->tau; st->rows_lo = sum; } else { st->hi = st->tau; }
        st->step = step + 1;
        st->tau = (step + 1 < iterations) ? 0.5f * (st->lo + st->hi) : st->lo;
    } else {
        // the final launch ran at lo
        st->rows_lo = bad ? -1 : sum;
    }
    if (tau_out) *tau_out = st->lo;
    if (rows_out) *rows_out = st->rows_lo;
}

hipError_t launch_gsc_budget(GscMergeArgs a, long long budget_rows, float tau_lo, float tau_hi, int iterations,
                             float *tau_out, long long *rows_out, void *state, hipStream_t stream) {
    BudgetState *st = reinterpret_cast<BudgetState *>(state);
    hipLaunchKernelGGL(budget_init_kernel, dim3(1), dim3(1), 0, stream, st, tau_lo, tau_hi);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (iterations == 0) {
        // no probe: the final launch below runs at tau_lo
        hipLaunchKernelGGL(budget_init_kernel, dim3(1), dim3(1), 0, stream, st, tau_lo, tau_lo);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    a.tau_dev = &st->tau;
    for (int it = 0; it <= iterations; ++it) {     // `iterations` probes, then the launch at the result
        // a probe only needs the row counts: clustering without reading the values, without the merge and
        // without writing rows (where the fast path runs; elsewhere a probe is a full merge)
        a.count_only = it < iterations;
        e = launch_gsc_merge(a, stream);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(budget_update_kernel, dim3(1), dim3(256), 0, stream, st, a.comp_lens, a.B * a.Hkv, budget_rows,
                           iterations, tau_out, rows_out);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace sc
