// Parameters and constants shared by the sc_gsc_merge kernels (internal).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sc {

constexpr int kGscThreads = 256;
constexpr int kMaxChunksPerItem = 32;
constexpr float kBand = 1e-4f;   // fp32 cosine error for d <= 128 is < 2e-5; inside the band -> fp64
constexpr int kPcountMask = (1 << 30) - 1;   // low bits of a pcount entry: clusters of the chunk

// State of the threshold search of sc_gsc_merge_budget (device memory, behind the merge workspace).
struct BudgetState {
    float tau;            // threshold of the next sc_gsc_merge launch
    float lo, hi;         // bracket: lo is assumed to meet the budget, hi not to
    int step;
    long long rows_lo;    // rows at lo (-1 until lo itself has been probed)
    // what the update needs, filed once per call
    long long budget_rows;
    int iterations;
    float *tau_out;
    long long *rows_out;
    // a probe's (sequence, head) workgroups add up their rows here; the last of them moves the bracket
    unsigned int arrived;
    int bad;
    long long total;
};

// after a probe at st->tau with `sum` rows in all (`bad`: some head overflowed its capacity, which counts
// as over budget): move the bracket and choose the next threshold: another midpoint, or lo itself for the
// final launch.  After the final launch (step == iterations): file the rows it produced.  One thread.
__device__ __forceinline__ void budget_bracket_step(BudgetState *st, long long sum, bool bad) {
    const int step = st->step;
    if (step < st->iterations) {
        const bool fits = !bad && sum <= st->budget_rows;
        if (fits) { st->lo = st->tau; st->rows_lo = sum; } else { st->hi = st->tau; }
        st->step = step + 1;
        st->tau = (step + 1 < st->iterations) ? 0.5f * (st->lo + st->hi) : st->lo;
    } else {
        st->rows_lo = bad ? -1 : sum;   // the final launch ran at lo
    }
    if (st->tau_out) *st->tau_out = st->lo;
    if (st->rows_out) *st->rows_out = st->rows_lo;
}

// A counting probe ends in the scan kernel, one workgroup per (sequence, head); with a search attached each
// of them adds its row count to the state and the last one to arrive moves the bracket, so no further
// launch is needed between two probes.  rows < 0: the head overflowed (or has no valid chunking).  One thread.
__device__ __forceinline__ void budget_probe_arrive(BudgetState *st, int rows, unsigned int n_heads) {
    if (rows >= 0) atomicAdd(reinterpret_cast<unsigned long long *>(&st->total), (unsigned long long)rows);
    else atomicOr(&st->bad, 1);
    __threadfence();
    if (atomicAdd(&st->arrived, 1u) == n_heads - 1u) {
        __threadfence();
        const long long sum = (long long)atomicAdd(reinterpret_cast<unsigned long long *>(&st->total), 0ull);
        const bool bad = atomicOr(&st->bad, 0) != 0;
        st->total = 0;
        st->bad = 0;
        st->arrived = 0u;
        budget_bracket_step(st, sum, bad);
    }
}

struct GscParams {
    const void *K, *V;
    int64_t stride_b, stride_h, stride_n;
    const int32_t *seq_lens, *offsets;
    int64_t offsets_stride_b;
    const int32_t *num_chunks;
    int B, Hkv, N_max;
    float tau;
    const float *tau_dev;   // if not NULL the threshold is read from device memory instead (budget search)
    BudgetState *budget;    // if not NULL: a counting probe of the budget search, see budget_probe_arrive
    void *Kc, *Vc;
    int out_is_bf16;
    int cap;
    int32_t *counts, *comp_lens;
    const int32_t *base_lens;   // [B, Hkv] rows already in Kc/Vc/counts (append mode), or NULL for none
    int32_t *cid;         // [B, Hkv, N_max]   cluster index of every token (caller's buffer or workspace)
    int32_t *cluster_id;  // the caller's buffer, or NULL if not requested
    int32_t *seedrow;     // [B, Hkv, N_max]   seed positions of a chunk that spans several blocks
    int32_t *pcount;      // [B, Hkv, N_max + 1] clusters per chunk (+ flag bit 30)
    int32_t *rowbase;     // [B, Hkv, N_max + 2] first output row of every chunk
    void *ktmp;           // [B, Hkv, N_max, d] merged keys at provisional rows (fast path)
    void *vtmp;           // [B, Hkv, N_max, d] merged values at provisional rows (fast path)
    int32_t *stmp;        // [B, Hkv, N_max]   cluster sizes at provisional rows (fast path)
    int count_only;       // fast path: cluster and count only (per-chunk cluster counts and comp_lens); no values are read, no rows written
    int chunks_per_item;
    int grid_x;           // fast path: workgroups per pass and (sequence, head) of the compress kernel
};

// rows already present in the outputs of (sequence, head) bh; an overflowed or impossible state counts as
// a full cache, so that nothing more is written and the new length is filed as -1
__device__ __forceinline__ int gsc_base_rows(const GscParams &p, int64_t bh, bool &bad) {
    const int raw = p.base_lens ? p.base_lens[bh] : 0;
    bad = raw < 0 || raw > p.cap;
    return bad ? p.cap : raw;
}

hipError_t launch_gsc_scan(const GscParams &p, hipStream_t stream);
hipError_t launch_gsc_fast(const GscParams &p, hipStream_t stream);

}  // namespace sc
