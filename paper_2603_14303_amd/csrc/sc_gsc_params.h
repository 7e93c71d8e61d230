// Parameters and constants shared by the sc_gsc_merge kernels (internal).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sc {

constexpr int kGscThreads = 256;
constexpr int kMaxChunksPerItem = 32;
constexpr float kBand = 1e-4f;   // fp32 cosine error for d <= 128 is < 2e-5; inside the band -> fp64
constexpr int kPcountMask = (1 << 30) - 1;   // low bits of a pcount entry: clusters of the chunk

struct GscParams {
    const void *K, *V;
    int64_t stride_b, stride_h, stride_n;
    const int32_t *seq_lens, *offsets;
    int64_t offsets_stride_b;
    const int32_t *num_chunks;
    int B, Hkv, N_max;
    float tau;
    const float *tau_dev;   // if not NULL the threshold is read from device memory instead (budget search)
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
