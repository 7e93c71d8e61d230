// sc_decode_attn: Proportional Attention for one decode step (paper Sec. 2.4, Eq. 4):
//     O = softmax(q K_c^T * scale + ln s) V_c   per (sequence, query head), GQA-grouped.
//
// Split-K: the rows of one (sequence, KV head) are cut into S contiguous ranges, one workgroup each;
// the G query heads that share the KV head are handled together so K_c/V_c are read once.  Inside a
// workgroup a row is spread over d/8 neighbouring lanes (16-byte pieces, fully coalesced); a wave
// loads 4 x (64/(d/8)) rows per step, forms the G dot products per row with a DPP all-reduce, and
// keeps an online softmax (running max, running sum, fp32 accumulator) per lane group.  Partials are
// merged through LDS, written to the workspace, and the workgroup that arrives last (ticket counter)
// folds the S partials into O.  The ticket is reset by that workgroup, so a workspace that was
// zeroed once stays ready for the next call.
#include "sc_device.h"
#include "sc_host.h"

namespace sc {

constexpr int kDecThreads = 256;
constexpr int kDecWaves = kDecThreads / kWave;
constexpr int kDecUnroll = 4;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr int kDecMaxSplits = 256;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

struct DecParams {
    const void *Q;
    int q_is_bf16;
    const void *Kc, *Vc;
    int cap;
    const int32_t *counts, *comp_lens;
    int B, Hq, Hkv;
    float scale_log2;     // scale * log2(e)
    void *O;
    int o_is_bf16;
    float *lse;
    int32_t *tickets;     // [B*Hkv], zero between calls
    float *part;          // [B*Hkv][S][G][D + 2]
    int max_splits, min_rows;
};

__device__ __forceinline__ int splits_for(int rows, int max_splits, int min_rows) {
    int s = (rows + min_rows - 1) / min_rows;
    return s < 1 ? 1 : (s > max_splits ? max_splits : s);
}

template <typename T, int D, int G>
__global__ __launch_bounds__(kDecThreads) void decode_kernel(DecParams p) {
    constexpr int LPR = D / 8;
    constexpr int RPW = kWave / LPR;
    constexpr int kRowsPerWaveStep = RPW * kDecUnroll;
    constexpr int kRowsPerBlockStep = kRowsPerWaveStep * kDecWaves;
    constexpr int kStride = D + 2;   // floats per (split, head) partial: acc[D], m, l

    __shared__ float s_acc[kDecWaves][G][D];
    __shared__ float s_m[kDecWaves][G];
    __shared__ float s_l[kDecWaves][G];
    __shared__ int s_last;

    const int split = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);   // scalar: keeps the row loop wave-uniform
    const int g = lane / LPR, c = lane % LPR;
    const int64_t bh = (int64_t)b * p.Hkv + h;
    const int rows_total = min(max(p.comp_lens[bh], 0), p.cap);
    const int S = splits_for(rows_total, p.max_splits, p.min_rows);
    if (split >= S) return;
    // contiguous row range of this split, a multiple of the block step except for the last one
    int per = (rows_total + S - 1) / S;
    per = (per + kRowsPerBlockStep - 1) / kRowsPerBlockStep * kRowsPerBlockStep;
    const int r0 = min(split * per, rows_total), r1 = min(r0 + per, rows_total);

    const T *Kbh = reinterpret_cast<const T *>(p.Kc) + bh * (int64_t)p.cap * D;
    const T *Vbh = reinterpret_cast<const T *>(p.Vc) + bh * (int64_t)p.cap * D;
    const int32_t *cnt_bh = p.counts + bh * (int64_t)p.cap;

    // query pieces of the G heads, pre-multiplied by scale*log2(e)
    float q[G][8];
#pragma unroll
    for (int hh = 0; hh < G; ++hh) {
        const int64_t qoff = ((int64_t)b * p.Hq + (int64_t)h * G + hh) * D + 8 * c;
        if (p.q_is_bf16) load8(reinterpret_cast<const bf16_t *>(p.Q) + qoff, q[hh]);
        else load8(reinterpret_cast<const float *>(p.Q) + qoff, q[hh]);
#pragma unroll
        for (int e = 0; e < 8; ++e) q[hh][e] *= p.scale_log2;
    }

    float acc[G][8], m[G], lsum[G];
#pragma unroll
    for (int hh = 0; hh < G; ++hh) {
        m[hh] = -INFINITY;
        lsum[hh] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[hh][e] = 0.f;
    }

    for (int base = r0 + wave * kRowsPerWaveStep; base < r1; base += kRowsPerBlockStep) {
        float kk[kDecUnroll][8], vv[kDecUnroll][8];
        float bias[kDecUnroll];
        bool ok[kDecUnroll];
#pragma unroll
        for (int u = 0; u < kDecUnroll; ++u) {
            const int row = base + u * RPW + g;
            ok[u] = row < r1;
            if (ok[u]) {
                load8(Kbh + (int64_t)row * D + 8 * c, kk[u]);
                load8(Vbh + (int64_t)row * D + 8 * c, vv[u]);
                bias[u] = __log2f((float)cnt_bh[row]);
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) { kk[u][e] = 0.f; vv[u][e] = 0.f; }
                bias[u] = 0.f;
            }
        }
#pragma unroll
        for (int hh = 0; hh < G; ++hh) {
            float s[kDecUnroll];
            float mx = m[hh];
#pragma unroll
            for (int u = 0; u < kDecUnroll; ++u) {
                float d = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) d = fmaf(q[hh][e], kk[u][e], d);
                d = row_allreduce_sum<LPR>(d);
                s[u] = ok[u] ? d + bias[u] : -INFINITY;
                mx = fmaxf(mx, s[u]);
            }
            const float m_safe = (mx == -INFINITY) ? 0.f : mx;
            const float alpha = fast_exp2(m[hh] - m_safe);
            m[hh] = mx;
            float pw[kDecUnroll];
            float psum = 0.f;
#pragma unroll
            for (int u = 0; u < kDecUnroll; ++u) {
                pw[u] = fast_exp2(s[u] - m_safe);
                psum += pw[u];
            }
            lsum[hh] = lsum[hh] * alpha + psum;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float a = acc[hh][e] * alpha;
#pragma unroll
                for (int u = 0; u < kDecUnroll; ++u) a = fmaf(pw[u], vv[u][e], a);
                acc[hh][e] = a;
            }
        }
    }

    // ---- fold the RPW lane groups of the wave (each saw different rows)
#pragma unroll
    for (int hh = 0; hh < G; ++hh) {
        float mw = m[hh];
#pragma unroll
        for (int off = LPR; off < kWave; off <<= 1) mw = fmaxf(mw, __shfl_xor(mw, off, kWave));
        const float m_safe = (mw == -INFINITY) ? 0.f : mw;
        const float f = fast_exp2(m[hh] - m_safe);
        float lw = lsum[hh] * f;
#pragma unroll
        for (int off = LPR; off < kWave; off <<= 1) lw += __shfl_xor(lw, off, kWave);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float a = acc[hh][e] * f;
#pragma unroll
            for (int off = LPR; off < kWave; off <<= 1) a += __shfl_xor(a, off, kWave);
            acc[hh][e] = a;
        }
        if (g == 0) {
#pragma unroll
            for (int e = 0; e < 8; ++e) s_acc[wave][hh][8 * c + e] = acc[hh][e];
            if (c == 0) { s_m[wave][hh] = mw; s_l[wave][hh] = lw; }
        }
    }
    __syncthreads();

    // ---- fold the waves, write this split's partial
    float *part_bh = p.part + bh * (int64_t)p.max_splits * G * kStride;
    for (int i = tid; i < G * D; i += kDecThreads) {
        const int hh = i / D, e = i % D;
        float mw = -INFINITY;
#pragma unroll
        for (int w = 0; w < kDecWaves; ++w) mw = fmaxf(mw, s_m[w][hh]);
        const float m_safe = (mw == -INFINITY) ? 0.f : mw;
        float a = 0.f, l = 0.f;
#pragma unroll
        for (int w = 0; w < kDecWaves; ++w) {
            const float f = fast_exp2(s_m[w][hh] - m_safe);
            a = fmaf(s_acc[w][hh][e], f, a);
            l = fmaf(s_l[w][hh], f, l);
        }
        float *dst = part_bh + ((int64_t)split * G + hh) * kStride;
        dst[e] = a;
        if (e == 0) { dst[D] = mw; dst[D + 1] = l; }
    }

    // ---- the workgroup that arrives last combines all splits
    __threadfence();
    __syncthreads();
    if (tid == 0) {
        const int ticket = atomicAdd(p.tickets + bh, 1);
        s_last = (ticket == S - 1);
        if (ticket == S - 1) p.tickets[bh] = 0;   // ready for the next call
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();
    for (int i = tid; i < G * D; i += kDecThreads) {
        const int hh = i / D, e = i % D;
        float mw = -INFINITY;
        for (int s = 0; s < S; ++s)
            mw = fmaxf(mw, __builtin_nontemporal_load(part_bh + ((int64_t)s * G + hh) * kStride + D));
        const float m_safe = (mw == -INFINITY) ? 0.f : mw;
        float a = 0.f, l = 0.f;
        for (int s = 0; s < S; ++s) {
            const float *src = part_bh + ((int64_t)s * G + hh) * kStride;
            const float f = fast_exp2(__builtin_nontemporal_load(src + D) - m_safe);
            a = fmaf(__builtin_nontemporal_load(src + e), f, a);
            l = fmaf(__builtin_nontemporal_load(src + D + 1), f, l);
        }
        const float out = (l > 0.f) ? a / l : 0.f;
        const int64_t ooff = ((int64_t)b * p.Hq + (int64_t)h * G + hh) * D + e;
        if (p.o_is_bf16) reinterpret_cast<uint16_t *>(p.O)[ooff] = (uint16_t)f32_to_bf16(out);
        else reinterpret_cast<float *>(p.O)[ooff] = out;
        if (e == 0 && p.lse) p.lse[(int64_t)b * p.Hq + (int64_t)h * G + hh] = (l > 0.f) ? (mw + __log2f(l)) * kLn2 : -INFINITY;
    }
}

__global__ void zero_words_kernel(int32_t *p, size_t n) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

size_t decode_workspace_state_bytes(int B, int Hkv) { return align_up((size_t)B * Hkv * 4, 256); }

static int clamp_splits() { return max(1, min(kDecMaxSplits, tuning().decode_max_splits)); }

size_t decode_workspace_bytes(int B, int Hq, int Hkv, int cap, int d) {
    (void)cap;
    const int G = Hq / Hkv;
    // sized for the largest split count the tuning knob may take, so the knob never invalidates a workspace
    return decode_workspace_state_bytes(B, Hkv) + align_up((size_t)B * Hkv * kDecMaxSplits * G * (d + 2) * 4, 256);
}

hipError_t launch_decode_init_workspace(void *ws, size_t state_bytes, hipStream_t stream) {
    const size_t n = state_bytes / 4;
    hipLaunchKernelGGL(zero_words_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream,
                       reinterpret_cast<int32_t *>(ws), n);
    return hipGetLastError();
}

template <typename T, int D, int G>
static hipError_t launch_g(const DecParams &p, hipStream_t stream) {
    const dim3 grid(p.max_splits, p.Hkv, p.B);
    hipLaunchKernelGGL((decode_kernel<T, D, G>), grid, dim3(kDecThreads), 0, stream, p);
    return hipGetLastError();
}

template <typename T, int D>
static hipError_t launch_td(const DecParams &p, int G, hipStream_t stream) {
    switch (G) {
        case 1: return launch_g<T, D, 1>(p, stream);
        case 2: return launch_g<T, D, 2>(p, stream);
        case 3: return launch_g<T, D, 3>(p, stream);
        case 4: return launch_g<T, D, 4>(p, stream);
        case 5: return launch_g<T, D, 5>(p, stream);
        case 6: return launch_g<T, D, 6>(p, stream);
        case 7: return launch_g<T, D, 7>(p, stream);
        case 8: return launch_g<T, D, 8>(p, stream);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_decode(const DecodeArgs &a, hipStream_t stream) {
    DecParams p;
    p.Q = a.Q; p.q_is_bf16 = a.q_dtype == DType::BF16;
    p.Kc = a.Kc; p.Vc = a.Vc; p.cap = a.cap;
    p.counts = a.counts; p.comp_lens = a.comp_lens;
    p.B = a.B; p.Hq = a.Hq; p.Hkv = a.Hkv;
    p.scale_log2 = a.scale * kLog2e;
    p.O = a.O; p.o_is_bf16 = a.o_dtype == DType::BF16;
    p.lse = a.lse;
    p.tickets = reinterpret_cast<int32_t *>(a.ws);
    p.part = reinterpret_cast<float *>(reinterpret_cast<char *>(a.ws) + decode_workspace_state_bytes(a.B, a.Hkv));
    p.min_rows = max(1, tuning().decode_min_rows);
    // never more splits than the capacity can feed
    const int by_cap = (a.cap + p.min_rows - 1) / p.min_rows;
    p.max_splits = max(1, min(clamp_splits(), by_cap));
    const int G = a.Hq / a.Hkv;
    if (a.kv_dtype == DType::BF16)
        return a.d == 128 ? launch_td<bf16_t, 128>(p, G, stream) : launch_td<bf16_t, 64>(p, G, stream);
    return a.d == 128 ? launch_td<float, 128>(p, G, stream) : launch_td<float, 64>(p, G, stream);
}

}  // namespace sc
