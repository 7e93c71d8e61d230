// C ABI of libsemanticache: argument validation on the host, then the kernel launchers.
// Everything that can be rejected without touching the device is rejected before any HIP call.
#include "../../include/semanticache.h"

#include <string.h>

#include "sc_host.h"
#include <vector>

namespace sc {

Tuning &tuning() {
    static Tuning t;
    return t;
}

static thread_local char g_last_error[256] = "";

static sc_status runtime_status(hipError_t e) {
    if (e == hipSuccess) return SC_OK;
    strncpy(g_last_error, hipGetErrorString(e), sizeof(g_last_error) - 1);
    g_last_error[sizeof(g_last_error) - 1] = 0;
    return SC_ERR_RUNTIME;
}

static bool dtype_ok(int t) { return t == SC_F32 || t == SC_BF16; }
static size_t elem_size(int t) { return t == SC_BF16 ? 2 : 4; }
static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static bool aligned4(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 3u) == 0; }

}  // namespace sc

using namespace sc;

extern "C" {

const char *sc_status_string(sc_status status) {
    switch (status) {
        case SC_OK: return "SC_OK";
        case SC_ERR_INVALID_ARG: return "SC_ERR_INVALID_ARG";
        case SC_ERR_UNSUPPORTED: return "SC_ERR_UNSUPPORTED";
        case SC_ERR_CAPACITY: return "SC_ERR_CAPACITY";
        case SC_ERR_WORKSPACE: return "SC_ERR_WORKSPACE";
        case SC_ERR_RUNTIME: return "SC_ERR_RUNTIME";
    }
    return "SC_ERR_UNKNOWN";
}

const char *sc_last_runtime_error(void) { return g_last_error; }

const char *sc_version(void) { return "0.1.0"; }

int sc_tune_set(const char *key, int value) {
    if (!key) return -1;
    Tuning &t = tuning();
    if (!strcmp(key, "decode_max_splits")) t.decode_max_splits = value;
    else if (!strcmp(key, "decode_min_rows")) t.decode_min_rows = value;
    else if (!strcmp(key, "decode_mfma_min_group")) t.decode_mfma_min_group = value;
    else if (!strcmp(key, "decode_local_handover")) t.decode_local_handover = value;
    else if (!strcmp(key, "decode_poll_budget")) t.decode_poll_budget = value;
    else if (!strcmp(key, "gsc_chunks_per_item")) t.gsc_chunks_per_item = value;
    else if (!strcmp(key, "gsc_grid_x")) t.gsc_grid_x = value;
    else if (!strcmp(key, "gsc_fast_path")) t.gsc_fast_path = value;
    else if (!strcmp(key, "gsc_chunks_per_task")) t.gsc_chunks_per_task = value;
    else if (!strcmp(key, "multi_block_rows")) t.multi_block_rows = value;
    else if (!strcmp(key, "multi_target_wgs")) t.multi_target_wgs = value;
    else return -1;
    return 0;
}

int sc_tune_get(const char *key) {
    if (!key) return -1;
    const Tuning &t = tuning();
    if (!strcmp(key, "decode_max_splits")) return t.decode_max_splits;
    if (!strcmp(key, "decode_min_rows")) return t.decode_min_rows;
    if (!strcmp(key, "decode_mfma_min_group")) return t.decode_mfma_min_group;
    if (!strcmp(key, "decode_local_handover")) return t.decode_local_handover;
    if (!strcmp(key, "decode_poll_budget")) return t.decode_poll_budget;
    if (!strcmp(key, "gsc_chunks_per_item")) return t.gsc_chunks_per_item;
    if (!strcmp(key, "gsc_grid_x")) return t.gsc_grid_x;
    if (!strcmp(key, "gsc_fast_path")) return t.gsc_fast_path;
    if (!strcmp(key, "gsc_chunks_per_task")) return t.gsc_chunks_per_task;
    if (!strcmp(key, "multi_block_rows")) return t.multi_block_rows;
    if (!strcmp(key, "multi_target_wgs")) return t.multi_target_wgs;
    return -1;
}

// ------------------------------------------------------------------------------------------------
sc_status sc_check_lengths(const int32_t *lengths, int count, int *first_bad, void *stream) {
    if (!lengths || count <= 0 || !aligned4(lengths)) return SC_ERR_INVALID_ARG;
    if (first_bad) *first_bad = -1;
    std::vector<int32_t> host((size_t)count);
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e = hipMemcpyAsync(host.data(), lengths, (size_t)count * sizeof(int32_t), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) return runtime_status(e);
    for (int i = 0; i < count; ++i)
        if (host[i] < 0) {
            if (first_bad) *first_bad = i;
            return SC_ERR_CAPACITY;
        }
    return SC_OK;
}

// ------------------------------------------------------------------------------------------------
sc_status sc_stream_read_probe(const void *src, size_t bytes, void *sink, void *stream) {
    if (!src || !sink || bytes < 16 || !aligned16(src) || !aligned4(sink)) return SC_ERR_INVALID_ARG;
    return runtime_status(launch_stream_read_probe(src, bytes, sink, static_cast<hipStream_t>(stream)));
}

// ------------------------------------------------------------------------------------------------
size_t sc_segment_workspace_bytes(int B, int N_max) {
    (void)B; (void)N_max;
    return 0;
}

sc_status sc_segment(const uint8_t *mask, int64_t mask_stride_b, const int32_t *seq_lens, int B, int N_max,
                     int32_t *offsets, int64_t offsets_stride_b, int offsets_cap, int32_t *num_chunks,
                     void *ws, size_t ws_bytes, void *stream) {
    (void)ws; (void)ws_bytes;
    if (!mask || !offsets || !num_chunks) return SC_ERR_INVALID_ARG;
    if (B <= 0 || N_max <= 0) return SC_ERR_INVALID_ARG;
    if (offsets_cap < 2) return SC_ERR_CAPACITY;
    if (mask_stride_b < N_max || offsets_stride_b < offsets_cap) return SC_ERR_INVALID_ARG;
    if (!aligned4(offsets) || !aligned4(num_chunks) || (seq_lens && !aligned4(seq_lens))) return SC_ERR_INVALID_ARG;
    if (B > 65535 * 32 || (N_max + 32767) / 32768 > 65535) return SC_ERR_UNSUPPORTED;   // grid sizes
    return runtime_status(launch_segment(mask, mask_stride_b, seq_lens, B, N_max, offsets, offsets_stride_b,
                                         offsets_cap, num_chunks, static_cast<hipStream_t>(stream)));
}

// ------------------------------------------------------------------------------------------------
size_t sc_gsc_merge_workspace_bytes(int B, int Hkv, int N_max, int d) {
    if (B <= 0 || Hkv <= 0 || N_max <= 0) return 0;
    return gsc_merge_workspace_bytes(B, Hkv, N_max, d);
}
size_t sc_gsc_merge_workspace_bytes_for(int B, int Hkv, int N_max, int d, sc_dtype out_dtype) {
    if (B <= 0 || Hkv <= 0 || N_max <= 0 || !dtype_ok(out_dtype)) return 0;
    return gsc_merge_workspace_bytes(B, Hkv, N_max, d, (int)elem_size(out_dtype));
}

static sc_status gsc_check_and_fill(const void *K, const void *V, sc_dtype in_dtype, int64_t stride_b, int64_t stride_h,
                                    int64_t stride_n, const int32_t *seq_lens, const int32_t *offsets,
                                    int64_t offsets_stride_b, const int32_t *num_chunks, int B, int Hkv, int N_max, int d,
                                    float tau, void *Kc, void *Vc, sc_dtype out_dtype, int cap, int32_t *counts,
                                    const int32_t *base_lens, bool append, int32_t *comp_lens, int32_t *cluster_id,
                                    void *ws, size_t ws_bytes, GscMergeArgs &a) {
    if (!K || !V || !offsets || !num_chunks || !Kc || !Vc || !counts || !comp_lens) return SC_ERR_INVALID_ARG;
    // every workgroup reads the old length while one of them files the new one
    if (append && (!base_lens || base_lens == comp_lens || !aligned4(base_lens))) return SC_ERR_INVALID_ARG;
    if (B <= 0 || Hkv <= 0 || N_max <= 0) return SC_ERR_INVALID_ARG;
    if (cap <= 0) return SC_ERR_CAPACITY;
    if (!dtype_ok(in_dtype) || !dtype_ok(out_dtype)) return SC_ERR_UNSUPPORTED;
    if (d != 64 && d != 128) return SC_ERR_UNSUPPORTED;
    if (Hkv > 65535 || B > 65535 || (long long)B * Hkv > (1 << 24)) return SC_ERR_UNSUPPORTED;   // grid sizes
    const size_t es = elem_size(in_dtype);
    if (stride_n < d || stride_h < 0 || stride_b < 0) return SC_ERR_INVALID_ARG;
    if ((stride_n * es) % 16 || (stride_h * es) % 16 || (stride_b * es) % 16) return SC_ERR_INVALID_ARG;
    if (!aligned16(K) || !aligned16(V) || !aligned16(Kc) || !aligned16(Vc)) return SC_ERR_INVALID_ARG;
    if (!aligned4(counts) || !aligned4(comp_lens) || !aligned4(offsets) || !aligned4(num_chunks)) return SC_ERR_INVALID_ARG;
    if (offsets_stride_b < 2) return SC_ERR_INVALID_ARG;
    if (tau != tau) return SC_ERR_INVALID_ARG;
    const size_t need = gsc_merge_workspace_bytes(B, Hkv, N_max, d, (int)elem_size(out_dtype));
    if (!ws || ws_bytes < need || (reinterpret_cast<uintptr_t>(ws) & 255u)) return SC_ERR_WORKSPACE;

    a.K = K; a.V = V; a.in_dtype = static_cast<DType>(in_dtype);
    a.stride_b = stride_b; a.stride_h = stride_h; a.stride_n = stride_n;
    a.seq_lens = seq_lens; a.offsets = offsets; a.offsets_stride_b = offsets_stride_b; a.num_chunks = num_chunks;
    a.B = B; a.Hkv = Hkv; a.N_max = N_max; a.d = d; a.tau = tau;
    a.Kc = Kc; a.Vc = Vc; a.out_dtype = static_cast<DType>(out_dtype); a.cap = cap;
    a.counts = counts; a.comp_lens = comp_lens; a.cluster_id = cluster_id; a.ws = ws;
    a.base_lens = append ? base_lens : nullptr;
    return SC_OK;
}

static sc_status gsc_common(const void *K, const void *V, sc_dtype in_dtype, int64_t stride_b, int64_t stride_h,
                            int64_t stride_n, const int32_t *seq_lens, const int32_t *offsets, int64_t offsets_stride_b,
                            const int32_t *num_chunks, int B, int Hkv, int N_max, int d, float tau, void *Kc, void *Vc,
                            sc_dtype out_dtype, int cap, int32_t *counts, const int32_t *base_lens, bool append,
                            int32_t *comp_lens, int32_t *cluster_id, void *ws, size_t ws_bytes, void *stream) {
    GscMergeArgs a;
    const sc_status st = gsc_check_and_fill(K, V, in_dtype, stride_b, stride_h, stride_n, seq_lens, offsets, offsets_stride_b,
                                            num_chunks, B, Hkv, N_max, d, tau, Kc, Vc, out_dtype, cap, counts, base_lens,
                                            append, comp_lens, cluster_id, ws, ws_bytes, a);
    if (st != SC_OK) return st;
    return runtime_status(launch_gsc_merge(a, static_cast<hipStream_t>(stream)));
}

sc_status sc_gsc_merge(const void *K, const void *V, sc_dtype in_dtype, int64_t stride_b, int64_t stride_h,
                       int64_t stride_n, const int32_t *seq_lens, const int32_t *offsets, int64_t offsets_stride_b,
                       const int32_t *num_chunks, int B, int Hkv, int N_max, int d, float tau, void *Kc, void *Vc,
                       sc_dtype out_dtype, int cap, int32_t *counts, int32_t *comp_lens, int32_t *cluster_id,
                       void *ws, size_t ws_bytes, void *stream) {
    return gsc_common(K, V, in_dtype, stride_b, stride_h, stride_n, seq_lens, offsets, offsets_stride_b, num_chunks, B, Hkv,
                      N_max, d, tau, Kc, Vc, out_dtype, cap, counts, nullptr, false, comp_lens, cluster_id, ws, ws_bytes,
                      stream);
}

sc_status sc_gsc_merge_append(const void *K, const void *V, sc_dtype in_dtype, int64_t stride_b, int64_t stride_h,
                              int64_t stride_n, const int32_t *seq_lens, const int32_t *offsets,
                              int64_t offsets_stride_b, const int32_t *num_chunks, int B, int Hkv, int N_max, int d,
                              float tau, void *Kc, void *Vc, sc_dtype out_dtype, int cap, int32_t *counts,
                              const int32_t *base_lens, int32_t *comp_lens, int32_t *cluster_id, void *ws,
                              size_t ws_bytes, void *stream) {
    return gsc_common(K, V, in_dtype, stride_b, stride_h, stride_n, seq_lens, offsets, offsets_stride_b, num_chunks, B, Hkv,
                      N_max, d, tau, Kc, Vc, out_dtype, cap, counts, base_lens, true, comp_lens, cluster_id, ws, ws_bytes,
                      stream);
}

size_t sc_gsc_merge_global_workspace_bytes(int B, int Hkv, int N_max, int d) {
    if (B <= 0 || Hkv <= 0 || N_max <= 0) return 0;
    return gsc_global_workspace_bytes(B, Hkv, N_max, d);
}

sc_status sc_gsc_merge_global(const void *K, const void *V, sc_dtype in_dtype, int64_t stride_b, int64_t stride_h,
                              int64_t stride_n, const int32_t *seq_lens, int B, int Hkv, int N_max, int d, float tau,
                              void *Kc, void *Vc, sc_dtype out_dtype, int cap, int32_t *counts, int32_t *comp_lens,
                              int32_t *cluster_id, void *ws, size_t ws_bytes, void *stream) {
    if (B <= 0 || Hkv <= 0 || N_max <= 0) return SC_ERR_INVALID_ARG;
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u)) return SC_ERR_WORKSPACE;
    // the start of the workspace takes the one-chunk offsets; everything else is checked as for sc_gsc_merge
    int32_t *offsets = reinterpret_cast<int32_t *>(ws), *num_chunks = offsets + 2 * B;
    GscMergeArgs a;
    const sc_status st = gsc_check_and_fill(K, V, in_dtype, stride_b, stride_h, stride_n, seq_lens, offsets, 2, num_chunks, B, Hkv,
                                            N_max, d, tau, Kc, Vc, out_dtype, cap, counts, nullptr, false, comp_lens, cluster_id,
                                            ws, ws_bytes, a);
    if (st != SC_OK) return st;
    if (ws_bytes < gsc_global_workspace_bytes(B, Hkv, N_max, d)) return SC_ERR_WORKSPACE;
    return runtime_status(launch_gsc_global(a, static_cast<hipStream_t>(stream)));
}

size_t sc_gsc_merge_budget_workspace_bytes(int B, int Hkv, int N_max, int d) {
    if (B <= 0 || Hkv <= 0 || N_max <= 0) return 0;
    return align_up(gsc_merge_workspace_bytes(B, Hkv, N_max, d), 256) + gsc_budget_state_bytes();
}

sc_status sc_gsc_merge_budget(const void *K, const void *V, sc_dtype in_dtype, int64_t stride_b, int64_t stride_h,
                              int64_t stride_n, const int32_t *seq_lens, const int32_t *offsets,
                              int64_t offsets_stride_b, const int32_t *num_chunks, int B, int Hkv, int N_max, int d,
                              int64_t budget_rows, float tau_lo, float tau_hi, int iterations, void *Kc, void *Vc,
                              sc_dtype out_dtype, int cap, int32_t *counts, int32_t *comp_lens, int32_t *cluster_id,
                              float *tau_out, int64_t *rows_out, void *ws, size_t ws_bytes, void *stream) {
    if (!tau_out || !aligned4(tau_out) || (rows_out && (reinterpret_cast<uintptr_t>(rows_out) & 7u))) return SC_ERR_INVALID_ARG;
    if (iterations < 0 || iterations > 32 || budget_rows < 0) return SC_ERR_INVALID_ARG;
    if (tau_lo != tau_lo || tau_hi != tau_hi || tau_lo > tau_hi) return SC_ERR_INVALID_ARG;
    if (B <= 0 || Hkv <= 0 || N_max <= 0) return SC_ERR_INVALID_ARG;
    // everything else is checked exactly as for sc_gsc_merge (no launch happens on a failed check)
    GscMergeArgs a;
    const sc_status st = gsc_check_and_fill(K, V, in_dtype, stride_b, stride_h, stride_n, seq_lens, offsets, offsets_stride_b,
                                            num_chunks, B, Hkv, N_max, d, tau_lo, Kc, Vc, out_dtype, cap, counts, nullptr,
                                            false, comp_lens, cluster_id, ws, ws_bytes, a);
    if (st != SC_OK) return st;
    const size_t gsc_bytes = align_up(gsc_merge_workspace_bytes(B, Hkv, N_max, d), 256);
    if (ws_bytes < gsc_bytes + gsc_budget_state_bytes()) return SC_ERR_WORKSPACE;
    return runtime_status(launch_gsc_budget(a, (long long)budget_rows, tau_lo, tau_hi, iterations, tau_out,
                                            reinterpret_cast<long long *>(rows_out),
                                            reinterpret_cast<char *>(ws) + gsc_bytes, static_cast<hipStream_t>(stream)));
}

// ------------------------------------------------------------------------------------------------
size_t sc_decode_attn_workspace_bytes(int B, int Hq, int Hkv, int cap, int d) {
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || cap <= 0 || Hq % Hkv) return 0;
    return decode_workspace_bytes(B, Hq, Hkv, cap, d);
}

sc_status sc_decode_attn_init_workspace(void *ws, size_t ws_bytes, int B, int Hkv, void *stream) {
    if (B <= 0 || Hkv <= 0) return SC_ERR_INVALID_ARG;
    const size_t state = decode_workspace_state_bytes(B, Hkv);
    if (!ws || ws_bytes < state || (reinterpret_cast<uintptr_t>(ws) & 255u)) return SC_ERR_WORKSPACE;
    return runtime_status(launch_decode_init_workspace(ws, state, static_cast<hipStream_t>(stream)));
}

static sc_status decode_common(const void *Q, sc_dtype q_dtype, const void *Kc, const void *Vc, sc_dtype kv_dtype, int cap,
                               const int32_t *counts, const int32_t *comp_lens, const void *Kt, const void *Vt,
                               int tail_cap, const int32_t *tail_lens, bool with_tail, int B, int Hq, int Hkv, int d,
                               float scale, void *O, sc_dtype o_dtype, float *lse, void *ws, size_t ws_bytes,
                               void *stream, size_t state_bytes = 0) {
    if (!Q || !Kc || !Vc || !counts || !comp_lens || !O) return SC_ERR_INVALID_ARG;
    if (with_tail && (!Kt || !Vt || !tail_lens)) return SC_ERR_INVALID_ARG;
    if (B <= 0 || Hq <= 0 || Hkv <= 0) return SC_ERR_INVALID_ARG;
    if (cap <= 0 || (with_tail && tail_cap <= 0)) return SC_ERR_CAPACITY;
    if (with_tail && (int64_t)cap + tail_cap > INT32_MAX) return SC_ERR_CAPACITY;
    if (!dtype_ok(q_dtype) || !dtype_ok(kv_dtype) || !dtype_ok(o_dtype)) return SC_ERR_UNSUPPORTED;
    if (d != 64 && d != 128) return SC_ERR_UNSUPPORTED;
    if (Hq % Hkv) return SC_ERR_UNSUPPORTED;
    if (Hq / Hkv > 8) return SC_ERR_UNSUPPORTED;
    if (Hkv > 65535 || B > 65535) return SC_ERR_UNSUPPORTED;
    if (!aligned16(Q) || !aligned16(Kc) || !aligned16(Vc) || !aligned16(O)) return SC_ERR_INVALID_ARG;
    if (with_tail && (!aligned16(Kt) || !aligned16(Vt) || !aligned4(tail_lens))) return SC_ERR_INVALID_ARG;
    if (!aligned4(counts) || !aligned4(comp_lens) || (lse && !aligned4(lse))) return SC_ERR_INVALID_ARG;
    if (scale != scale) return SC_ERR_INVALID_ARG;
    size_t need = decode_workspace_bytes(B, Hq, Hkv, cap, d);
    if (state_bytes) need = need - decode_workspace_state_bytes(B, Hkv) + state_bytes;
    if (!ws || ws_bytes < need || (reinterpret_cast<uintptr_t>(ws) & 255u)) return SC_ERR_WORKSPACE;

    DecodeArgs a;
    a.state_bytes = state_bytes;
    a.Q = Q; a.q_dtype = static_cast<DType>(q_dtype);
    a.Kc = Kc; a.Vc = Vc; a.kv_dtype = static_cast<DType>(kv_dtype); a.cap = cap;
    a.counts = counts; a.comp_lens = comp_lens;
    if (with_tail) { a.Kt = Kt; a.Vt = Vt; a.tail_lens = tail_lens; a.tail_cap = tail_cap; }
    a.B = B; a.Hq = Hq; a.Hkv = Hkv; a.d = d;
    a.scale = (scale == 0.f) ? 1.0f / sqrtf((float)d) : scale;
    a.O = O; a.o_dtype = static_cast<DType>(o_dtype); a.lse = lse; a.ws = ws;
    return runtime_status(launch_decode(a, static_cast<hipStream_t>(stream)));
}

sc_status sc_decode_attn(const void *Q, sc_dtype q_dtype, const void *Kc, const void *Vc, sc_dtype kv_dtype, int cap,
                         const int32_t *counts, const int32_t *comp_lens, int B, int Hq, int Hkv, int d, float scale,
                         void *O, sc_dtype o_dtype, float *lse, void *ws, size_t ws_bytes, void *stream) {
    return decode_common(Q, q_dtype, Kc, Vc, kv_dtype, cap, counts, comp_lens, nullptr, nullptr, 0, nullptr, false, B, Hq,
                         Hkv, d, scale, O, o_dtype, lse, ws, ws_bytes, stream);
}

sc_status sc_decode_attn_static(const void *Q, sc_dtype q_dtype, const void *Kc, const void *Vc, sc_dtype kv_dtype,
                                int cap, const int32_t *counts, const int32_t *comp_lens, int B, int Hq, int Hkv, int d,
                                float scale, void *O, sc_dtype o_dtype, float *lse, void *stream) {
    // the size check comes first: nothing below may depend on a scratch that is too small
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv) return SC_ERR_INVALID_ARG;
    if (cap <= 0) return SC_ERR_CAPACITY;
    if (d != 64 && d != 128) return SC_ERR_UNSUPPORTED;
    if (decode_workspace_bytes(B, Hq, Hkv, cap, d) > kDecodeStaticScratchBytes) return SC_ERR_WORKSPACE;
    if ((long long)B * Hkv > kDecodeStaticMaxHeads) return SC_ERR_WORKSPACE;
    if (!Q || !Kc || !Vc || !counts || !comp_lens || !O) return SC_ERR_INVALID_ARG;
    void *ws = nullptr;
    const hipError_t e = decode_static_scratch(&ws);
    if (e != hipSuccess) return runtime_status(e);
    // The array is shared by calls of every shape, so its state region (epochs and flags of the split
    // hand-over) has ONE layout, for kDecodeStaticMaxHeads heads: a call of one shape never writes partials
    // over the state a call of another shape relies on.  The partials follow behind it.
    return decode_common(Q, q_dtype, Kc, Vc, kv_dtype, cap, counts, comp_lens, nullptr, nullptr, 0, nullptr, false, B, Hq,
                         Hkv, d, scale, O, o_dtype, lse, ws, kDecodeStaticArrayBytes, stream, kDecodeStaticStateBytes);
}

sc_status sc_decode_attn_tail(const void *Q, sc_dtype q_dtype, const void *Kc, const void *Vc, sc_dtype kv_dtype, int cap,
                              const int32_t *counts, const int32_t *comp_lens, const void *Kt, const void *Vt,
                              int tail_cap, const int32_t *tail_lens, int B, int Hq, int Hkv, int d, float scale,
                              void *O, sc_dtype o_dtype, float *lse, void *ws, size_t ws_bytes, void *stream) {
    return decode_common(Q, q_dtype, Kc, Vc, kv_dtype, cap, counts, comp_lens, Kt, Vt, tail_cap, tail_lens, true, B, Hq,
                         Hkv, d, scale, O, o_dtype, lse, ws, ws_bytes, stream);
}

size_t sc_multi_attn_workspace_bytes(int B, int Hq, int Hkv, int nq, int cap, int d) {
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || nq <= 0 || cap <= 0 || Hq % Hkv) return 0;
    return multi_workspace_bytes(B, Hq, Hkv, nq, cap, d);
}

static sc_status multi_common(const void *Q, sc_dtype q_dtype, int nq, const void *Kc, const void *Vc, sc_dtype kv_dtype,
                              int cap, const int32_t *counts, const int32_t *comp_lens, const void *Kt, const void *Vt,
                              int tail_cap, const int32_t *tail_lens, int causal, bool with_tail, int B, int Hq, int Hkv,
                              int d, float scale, void *O, sc_dtype o_dtype, float *lse, void *ws, size_t ws_bytes,
                              void *stream) {
    if (!Q || !Kc || !Vc || !counts || !comp_lens || !O) return SC_ERR_INVALID_ARG;
    if (with_tail && (!Kt || !Vt || !tail_lens || !aligned16(Kt) || !aligned16(Vt) || !aligned4(tail_lens))) return SC_ERR_INVALID_ARG;
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || nq <= 0) return SC_ERR_INVALID_ARG;
    if (cap <= 0 || (with_tail && tail_cap <= 0)) return SC_ERR_CAPACITY;
    if (with_tail && (int64_t)cap + tail_cap > (1 << 30)) return SC_ERR_CAPACITY;
    // the mask between the query rows exists on the matrix-core path only
    if (with_tail && causal && !(d == 128 && q_dtype == SC_BF16 && kv_dtype == SC_BF16)) return SC_ERR_UNSUPPORTED;
    if (!dtype_ok(q_dtype) || !dtype_ok(kv_dtype) || !dtype_ok(o_dtype)) return SC_ERR_UNSUPPORTED;
    if (d != 64 && d != 128) return SC_ERR_UNSUPPORTED;
    if (Hq % Hkv) return SC_ERR_UNSUPPORTED;
    if (Hq / Hkv > 8) return SC_ERR_UNSUPPORTED;
    if (Hkv > 65535 || B > 65535 || nq > 4096) return SC_ERR_UNSUPPORTED;   // grid sizes
    if (!aligned16(Q) || !aligned16(Kc) || !aligned16(Vc) || !aligned4(O)) return SC_ERR_INVALID_ARG;
    if (!aligned4(counts) || !aligned4(comp_lens) || (lse && !aligned4(lse))) return SC_ERR_INVALID_ARG;
    if (scale != scale) return SC_ERR_INVALID_ARG;
    const size_t need = multi_workspace_bytes(B, Hq, Hkv, nq, cap + (with_tail ? tail_cap : 0), d);
    if (!ws || ws_bytes < need || (reinterpret_cast<uintptr_t>(ws) & 255u)) return SC_ERR_WORKSPACE;

    MultiArgs a;
    a.Q = Q; a.q_dtype = static_cast<DType>(q_dtype); a.nq = nq;
    a.Kc = Kc; a.Vc = Vc; a.kv_dtype = static_cast<DType>(kv_dtype); a.cap = cap;
    a.counts = counts; a.comp_lens = comp_lens;
    if (with_tail) { a.Kt = Kt; a.Vt = Vt; a.tail_lens = tail_lens; a.tail_cap = tail_cap; a.causal = causal ? 1 : 0; }
    a.B = B; a.Hq = Hq; a.Hkv = Hkv; a.d = d;
    a.scale = (scale == 0.f) ? 1.0f / sqrtf((float)d) : scale;
    a.O = O; a.o_dtype = static_cast<DType>(o_dtype); a.lse = lse; a.ws = ws;
    return runtime_status(launch_multi(a, static_cast<hipStream_t>(stream)));
}

sc_status sc_multi_attn(const void *Q, sc_dtype q_dtype, int nq, const void *Kc, const void *Vc, sc_dtype kv_dtype,
                        int cap, const int32_t *counts, const int32_t *comp_lens, int B, int Hq, int Hkv, int d,
                        float scale, void *O, sc_dtype o_dtype, float *lse, void *ws, size_t ws_bytes, void *stream) {
    return multi_common(Q, q_dtype, nq, Kc, Vc, kv_dtype, cap, counts, comp_lens, nullptr, nullptr, 0, nullptr, 0, false, B,
                        Hq, Hkv, d, scale, O, o_dtype, lse, ws, ws_bytes, stream);
}

sc_status sc_multi_attn_tail(const void *Q, sc_dtype q_dtype, int nq, const void *Kc, const void *Vc, sc_dtype kv_dtype,
                             int cap, const int32_t *counts, const int32_t *comp_lens, const void *Kt, const void *Vt,
                             int tail_cap, const int32_t *tail_lens, int causal, int B, int Hq, int Hkv, int d,
                             float scale, void *O, sc_dtype o_dtype, float *lse, void *ws, size_t ws_bytes, void *stream) {
    return multi_common(Q, q_dtype, nq, Kc, Vc, kv_dtype, cap, counts, comp_lens, Kt, Vt, tail_cap, tail_lens, causal, true,
                        B, Hq, Hkv, d, scale, O, o_dtype, lse, ws, ws_bytes, stream);
}

}  // extern "C"
