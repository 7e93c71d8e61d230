// Host-side launcher declarations (internal; the public boundary is include/semanticache.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace sc {

enum class DType : int { F32 = 0, BF16 = 1 };

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---- sc_segment
hipError_t launch_segment(const uint8_t *mask, int64_t mask_stride_b, const int32_t *seq_lens, int B, int n_max,
                          int32_t *offsets, int64_t offsets_stride_b, int offsets_cap, int32_t *num_chunks,
                          hipStream_t stream);

// ---- sc_gsc_merge
struct GscMergeArgs {
    const void *K, *V;
    DType in_dtype;
    int64_t stride_b, stride_h, stride_n;   // elements
    const int32_t *seq_lens, *offsets;
    int64_t offsets_stride_b;
    const int32_t *num_chunks;
    int B, Hkv, N_max, d;
    float tau;
    void *Kc, *Vc;
    DType out_dtype;
    int cap;
    int32_t *counts, *comp_lens, *cluster_id;
    const int32_t *base_lens = nullptr;   // append mode: rows already in the outputs, [B, Hkv]
    const float *tau_dev = nullptr;       // threshold in device memory (overrides tau)
    bool count_only = false;              // only comp_lens is produced (bf16 / d = 128 fast path; elsewhere the full merge runs)
    void *budget_state = nullptr;         // counting probe of the budget search: its scan kernel also moves the bracket (fast path only)
    void *ws;
};
// out_elem_bytes: element size of the merged rows the call will write (4 sizes it for either output type)
size_t gsc_merge_workspace_bytes(int B, int Hkv, int N_max, int d, int out_elem_bytes = 4);
hipError_t launch_gsc_merge(const GscMergeArgs &a, hipStream_t stream);
bool gsc_merge_takes_fast_path(const GscMergeArgs &a);

// ---- sc_gsc_merge_global: the whole sequence as one chunk (a.offsets / a.num_chunks are not used)
size_t gsc_global_workspace_bytes(int B, int Hkv, int N_max, int d);
hipError_t launch_gsc_global(const GscMergeArgs &a, hipStream_t stream);

// ---- sc_gsc_merge_budget: bisection on the threshold, all on the device
size_t gsc_budget_state_bytes();
hipError_t launch_gsc_budget(GscMergeArgs a, long long budget_rows, float tau_lo, float tau_hi, int iterations,
                             float *tau_out, long long *rows_out, void *state, hipStream_t stream);

// ---- sc_decode_attn
struct DecodeArgs {
    const void *Q;
    DType q_dtype;
    const void *Kc, *Vc;
    DType kv_dtype;
    int cap;
    const int32_t *counts, *comp_lens;
    const void *Kt = nullptr, *Vt = nullptr;   // uncompressed tail [B, Hkv, tail_cap, d], or none
    const int32_t *tail_lens = nullptr;
    int tail_cap = 0;
    int B, Hq, Hkv, d;
    float scale;
    void *O;
    DType o_dtype;
    float *lse;
    void *ws;
    size_t state_bytes = 0;   // size of the state region at the start of ws; 0 = decode_workspace_state_bytes(B, Hkv)
};
size_t decode_workspace_bytes(int B, int Hq, int Hkv, int cap, int d);
size_t decode_workspace_state_bytes(int B, int Hkv);
hipError_t launch_decode_init_workspace(void *ws, size_t state_bytes, hipStream_t stream);
hipError_t launch_decode(const DecodeArgs &a, hipStream_t stream);
// sc_decode_attn_static: device address of the current GPU's file-scope scratch array (looked up once per device)
constexpr size_t kDecodeStaticScratchBytes = (size_t)16 << 20;
constexpr int kDecodeStaticMaxHeads = 1024;   // (sequence, KV head) pairs its state region is laid out for, whatever the call's shape
constexpr size_t kDecodeStaticStateBytes = 256 + (size_t)kDecodeStaticMaxHeads * 520;   // = decode_workspace_state_bytes(1, 1024)
constexpr size_t kDecodeStaticArrayBytes = kDecodeStaticScratchBytes + kDecodeStaticStateBytes;
hipError_t decode_static_scratch(void **ptr);

// ---- sc_multi_attn
struct MultiArgs {
    const void *Q;            // [nq, B, Hq, d]
    DType q_dtype;
    int nq;
    const void *Kc, *Vc;
    DType kv_dtype;
    int cap;
    const int32_t *counts, *comp_lens;
    const void *Kt = nullptr, *Vt = nullptr;   // uncompressed tail [B, Hkv, tail_cap, d], or none
    const int32_t *tail_lens = nullptr;
    int tail_cap = 0;
    int causal = 0;           // the last nq tail rows are the query rows' own tokens
    int B, Hq, Hkv, d;
    float scale;
    void *O;                  // [nq, B, Hq, d]
    DType o_dtype;
    float *lse;               // [nq, B, Hq] or NULL
    void *ws;
};
size_t multi_workspace_bytes(int B, int Hq, int Hkv, int nq, int cap, int d);
hipError_t launch_multi(const MultiArgs &a, hipStream_t stream);
// matrix-core path alone (bf16, d = 128): partials in a.ws, no state
size_t multi_fast_workspace_bytes(int B, int Hq, int Hkv, int nq, int cap);
hipError_t launch_multi_fast(const MultiArgs &a, hipStream_t stream);

// ---- measuring aid: streaming read of a buffer
hipError_t launch_stream_read_probe(const void *src, size_t bytes, void *sink, hipStream_t stream);

// tuning knobs (read by the launchers; set through sc_tune_set)
struct Tuning {
    int decode_max_splits = 0;      // split-K workgroups per (sequence, KV head); <= 0 picks it from B*Hkv
    int decode_min_rows = 192;      // rows of the merged cache a split should at least get
    int decode_local_handover = 1;  // 0: split partials always go through memory, also when a head's splits share an XCC
    int decode_poll_budget = 1 << 20;   // polls (about 0.3 us each) of the folding workgroup before it gives up; negative: give up at once (host-driven test of the failure path)
    int decode_mfma_min_group = 9;  // query heads per KV head from which single-row decode runs on the multi-row kernel (9 = never)
    int gsc_chunks_per_item = 16;   // chunks handled by one workgroup work item
    int gsc_grid_x = 0;             // workgroups per pass and (sequence, KV head); <= 0 picks it from the sequence length
    int gsc_chunks_per_task = 0;    // fast path: chunks handled by one single-wave workgroup; <= 0: 2, or 1 for a call of a few thousand tokens
    int gsc_fast_path = 1;          // 0 forces the generic kernels even for bf16 / d = 128
    int multi_block_rows = 0;       // query rows per workgroup of sc_multi_attn: 16 or 32; <= 0 picks it from the shape of the call
    int multi_target_wgs = 256;     // workgroups the split count of sc_multi_attn aims at (one per compute unit)
};
Tuning &tuning();

}  // namespace sc
