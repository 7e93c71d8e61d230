// sc_decode_attn: Proportional Attention for one decode step (paper Sec. 2.4, Eq. 4):
//     O = softmax(q K_c^T * scale + ln s) V_c   per (sequence, query head), GQA-grouped.
// sc_decode_attn_tail: the same over the merged rows followed by an uncompressed tail of new tokens,
// which attend as clusters of one (ln 1 = 0).
//
// Split-K.  The rows of one (sequence, KV head) are cut into S contiguous ranges, one workgroup each;
// the G query heads that share the KV head are handled together so K_c/V_c are read once.  A row is
// spread over d/8 neighbouring lanes (16-byte pieces, fully coalesced), a wave-wide load covers
// 64/(d/8) rows, and one "step" of a wave is U such loads of K_c and of V_c; the next step's loads
// are requested as soon as the current step's registers are free.
//
// Fast kernel (bf16 cache and query, d = 128, up to 8 query heads per KV head; 12 wavefronts per
// workgroup).  Per step a wave takes 16 rows; both products run on the matrix cores, the scores after
// the wave has turned its key rows around through a small LDS tile, the output sums straight from the
// loaded value registers (see the comment inside the kernel).  Softmax is online, per head, in the exp2
// domain with a log2(size) bias.  Partials (running max, sum, fp32 sums) are folded across the
// wavefronts and written to the workspace; every split but the last then publishes a flag, the
// workgroup of the last split waits for the flags (bounded) and folds the S partials into O.  The
// hand-over is described above publish_or_collect below.
//
// Generic kernel (d = 64, fp32 caches or queries): same split-K scheme, plain DPP all-reduce.
#include <type_traits>
#include "sc_device.h"
#include "sc_host.h"

#include <mutex>

namespace sc {

constexpr int kDecThreads = 256;
constexpr int kDecWaves = kDecThreads / kWave;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr int kDecMaxSplits = 64;
constexpr int kDecUnroll = 4;   // loads per step of the generic kernel

typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef short dec_short4 __attribute__((ext_vector_type(4)));
typedef __bf16 dec_bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int dec_u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), c, false);
}

// LDS traffic of one wavefront executes in order; this only keeps the compiler from moving accesses to
// other lanes' data across the point where the lanes of a wave hand data to each other
__device__ __forceinline__ void wave_lds_handover() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

struct DecParams {
    const void *Q;
    int q_is_bf16;
    const void *Kc, *Vc;
    int cap;
    const int32_t *counts, *comp_lens;
    const void *Kt, *Vt;           // uncompressed tail [B, Hkv, tail_cap, D] (same element type), or NULL
    const int32_t *tail_lens;      // [B] tokens in the tail
    int tail_cap;
    int B, Hq, Hkv;
    float scale_log2;     // scale * log2(e)
    void *O;
    int o_is_bf16;
    float *lse;
    int32_t *status;      // workspace status word: 0, or -1 once a hand-over has failed
    struct HeadSync *sync;   // [B*Hkv] epoch and per-split flags of the hand-over
    float *part;          // [B*Hkv][max_splits][G][D + 4]
    int max_splits, min_rows;
    int local;            // all splits of a head share one XCC (see publish_or_collect)
    int poll_budget;      // polls of the folding workgroup before it gives up
};

__device__ __forceinline__ int splits_for(int rows, int max_splits, int min_rows) {
    int s = (rows + min_rows - 1) / min_rows;
    return s < 1 ? 1 : (s > max_splits ? max_splits : s);
}

// value of lane SRC of the own 16-lane row (ds_swizzle bit-mask mode: keep lane bit 4, force the low bits)
template <int SRC> __device__ __forceinline__ float row_bcast(float x) {
    return __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(x), 0x10 | (SRC << 5)));
}
template <int N, int I = 0> struct BcastAll {
    static __device__ __forceinline__ void run(float x, float (&out)[N]) {
        out[I] = row_bcast<I>(x);
        if constexpr (I + 1 < N) BcastAll<N, I + 1>::run(x, out);
    }
};


// ------------------------------------------------------------------------------------------------
// Hand-over of the split partials to the workgroup that folds them.
//
// Grid: one-dimensional, workgroup id = split * (B * Hkv) + (sequence, head).  The workgroup of the
// LAST split of a (sequence, head) folds; it has the highest id of its head, so everything it waits for
// was dispatched before it.  The wait is bounded all the same.
//
// Per (sequence, head) the workspace holds an epoch word and one 64-bit flag per split.  A split
// publishes by storing (epoch + 1) together with the number of the XCC (chiplet) it ran on; the folder
// accepts a flag only if it carries that value, and raises the epoch when it is done.  Flags therefore
// never need clearing and a flag left behind by an earlier call can never be taken for a current one.
//
// Every wavefront waits for its own partial stores to be acknowledged before the workgroup's barrier,
// and only then is the flag stored: the flag can never overtake a partial.
//
// Two ways of moving the partials:
//   local   (B * Hkv a multiple of 8)  the hardware hands workgroup ids to the 8 XCCs round robin, so
//           all splits of a head sit on ONE XCC and share its L2: plain stores, acknowledged by that L2,
//           and device-scope loads by the folder (they skip the reader's vector cache and are served by
//           the L2 that holds the lines).  The folder checks the XCC numbers in the flags against its
//           own; if they ever differed the partials might be invisible to it, and the call fails (below)
//           instead of folding them.
//   remote  (any other shape)  the splits of a head are spread over the XCCs, whose L2s are not coherent
//           with each other inside a kernel: partials are written through to memory (device-scope
//           stores) and read back with device-scope loads.
//
// Failure (the wait ran out, or XCC numbers differ in local mode): the head group's outputs are filled
// with NaN, the workspace's status word is set to -1 and the head's epoch is poisoned, so that every
// later call on this workspace also reports NaN for it until the workspace is initialised again.  A
// workgroup that publishes after the folder gave up can thus never feed a later call.
struct HeadSync {
    unsigned long long epoch;
    unsigned long long flag[kDecMaxSplits];
};
constexpr unsigned long long kEpochPoison = ~0ull;
constexpr size_t kDecStatusBytes = 256;   // the workspace starts with the status word (int32: 0, or -1 after a failure)

__device__ __forceinline__ int xcc_number() {
    // XCC_ID hardware register, bits [3:0]: the chiplet this wavefront runs on
    return __builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) & 0xF;
}
__device__ __forceinline__ void store_partial(float *p, float v, bool local) {
    if (local) *p = v;
    else __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Returns 0 in the workgroups that are done after publishing, 1 in the folding workgroup once every
// other split of the (sequence, head) is published, -1 there if the hand-over failed.
__device__ __forceinline__ int publish_or_collect(HeadSync *hs, unsigned long long epoch, int S, int split, int tid,
                                                  bool local, int poll_budget, int *s_flag) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wavefront's partial stores are acknowledged
    __syncthreads();
    const int xcc = xcc_number();
    const unsigned long long want = epoch + 1ull;
    if (split != S - 1) {
        if (tid == 0)
            __hip_atomic_store(&hs->flag[split], (want << 8) | (unsigned long long)(xcc + 1), __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        return 0;
    }
    if (tid < kWave) {
        int budget = poll_budget;
        bool all = S <= 1;   // a single split has nothing to wait for
        unsigned long long f0 = (unsigned long long)(xcc + 1), f1 = f0;
        while (!all && poll_budget >= 0) {   // a negative budget gives up without looking (host-driven test of the failure path)
            f0 = (tid < S - 1) ? __hip_atomic_load(&hs->flag[tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : (want << 8);
            f1 = (tid + kWave < S - 1) ? __hip_atomic_load(&hs->flag[tid + kWave], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : (want << 8);
            all = __ballot((f0 >> 8) == want && (f1 >> 8) == want) == ~0ull;
            budget = __builtin_amdgcn_readfirstlane(budget) - 1;
            if (all || budget < 0) break;
            __builtin_amdgcn_s_sleep(2);
        }
        // in local mode every published flag must name the folder's own XCC
        const bool same0 = (tid >= S - 1) || (int)(f0 & 0xFF) == xcc + 1;
        const bool same1 = (tid + kWave >= S - 1) || (int)(f1 & 0xFF) == xcc + 1;
        const bool same = __ballot(same0 && same1) == ~0ull;
        if (tid == 0) *s_flag = (all && (same || !local)) ? 1 : -1;
    }
    __syncthreads();
    return *s_flag;
}

// a failed hand-over: the outputs of the (sequence, head) say so, and so does the workspace from now on
template <int G, int D>
__device__ __forceinline__ void file_failure(const DecParams &p, HeadSync *hs, int b, int h, int tid, int nthreads) {
    const float bad = __builtin_nanf("");
    for (int i = tid; i < G * D; i += nthreads) {
        const int64_t ooff = ((int64_t)b * p.Hq + (int64_t)h * G + i / D) * D + i % D;
        if (p.o_is_bf16) reinterpret_cast<uint16_t *>(p.O)[ooff] = (uint16_t)0x7FC0;
        else reinterpret_cast<float *>(p.O)[ooff] = bad;
        if (i % D == 0 && p.lse) p.lse[(int64_t)b * p.Hq + (int64_t)h * G + i / D] = bad;
    }
    if (tid == 0) {
        __hip_atomic_store(p.status, -1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&hs->epoch, kEpochPoison, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

constexpr int kPartPad = 4;   // floats after the D accumulators of a partial: m, l, 2 unused (keeps 16-byte rows)

typedef unsigned int u32x4_dec_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2_dec_t __attribute__((ext_vector_type(2)));
constexpr int kAuxDeviceScope = 16;   // buffer-load cache policy: sc1 = device scope (skips the vector cache)
constexpr int kAuxStream = 2;         // buffer-load cache policy: nt = read once by this launch (the cache rows: a step reads each exactly once;
                                      // without the hint they displace the partials and flags from the caches: 10.3 -> 9.6 us on a 32k-token layer)

// ------------------------------------------------------------------------------------------------
// Fold the S split partials of one (sequence, KV head) into O; run by the workgroup of the last split.
// A thread owns one 16-byte piece of one head's output and every NS-th split.  Every wavefront finds the
// heads' maxima and denominators by itself, from the (m, l) pairs of all splits held two to eight per
// lane and reduced with lane exchanges, so nothing has to go through LDS before the weights are known.
// All loads of a pass (the pairs, up to KMAX partial pieces and their m) are requested before the first
// is used: the fold costs one trip to the partials, one barrier and one store.  s_red: NTHREADS * 4 floats.
template <int D, int G, int NTHREADS>
__device__ __forceinline__ void combine_splits(const DecParams &p, const float *part_bh, int S, int b, int h, int tid,
                                               float *s_red) {
    constexpr int kStride = D + kPartPad;
    constexpr int QPR = D / 4;                  // 16-byte pieces per partial row
    constexpr int COMBOS = G * QPR;             // (head, piece) pairs
    constexpr int NS = NTHREADS / COMBOS;       // split groups
    constexpr int KMAX = 6;                     // pieces in flight per thread and pass
    constexpr int GPW = G <= 1 ? 1 : (G <= 2 ? 2 : (G <= 4 ? 4 : 8));   // heads padded to a power of two
    constexpr int EPL = kDecMaxSplits * GPW / kWave;                    // (split, head) pairs per lane
    static_assert(NS >= 1 && EPL >= 1, "one thread per (head, piece) at least");
    const int lane = tid & (kWave - 1);
    const int sg = tid / COMBOS, rem = tid - sg * COMBOS;
    const int g = rem / QPR, q4 = rem - g * QPR;
    const bool worker = sg < NS;
    // the partials of this head behind a buffer descriptor: splits beyond S read as zeros
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(part_bh), (short)0,
                                                                        S * G * kStride * 4, 0x00020000);
    constexpr int kNowhere = 0x7FFFFFF0;        // an offset beyond any descriptor: the load returns zeros
    const int my_off = (g * kStride + 4 * q4) * 4;
    float4 x[KMAX];
    float xm[KMAX];
    auto load_pass = [&](int s0) {
#pragma unroll
        for (int k = 0; k < KMAX; ++k) {
            const int s = s0 + sg + NS * k;
            const bool ok = worker && s < S;
            const u32x4_dec_t t = __builtin_amdgcn_raw_buffer_load_b128(rs, ok ? my_off + s * (G * kStride * 4) : kNowhere, 0,
                                                                         kAuxDeviceScope);
            x[k] = make_float4(__uint_as_float(t.x), __uint_as_float(t.y), __uint_as_float(t.z), __uint_as_float(t.w));
            xm[k] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs, ok ? ((s * G + g) * kStride + D) * 4 : kNowhere, 0,
                                                                          kAuxDeviceScope));
        }
    };
    load_pass(0);
    // (m, l) of pair e = lane + 64 j: split e / GPW, head e % GPW = lane % GPW
    const int gl = lane % GPW;
    float em[EPL], el[EPL];
#pragma unroll
    for (int j = 0; j < EPL; ++j) {
        const int s = (lane + kWave * j) / GPW;
        const bool ok = s < S && gl < G;
        const u32x2_dec_t ml = __builtin_amdgcn_raw_buffer_load_b64(rs, ok ? ((s * G + gl) * kStride + D) * 4 : kNowhere, 0,
                                                                     kAuxDeviceScope);
        em[j] = ok ? __uint_as_float(ml.x) : -INFINITY;
        el[j] = ok ? __uint_as_float(ml.y) : 0.f;
    }
    float mx = em[0];
#pragma unroll
    for (int j = 1; j < EPL; ++j) mx = fmaxf(mx, em[j]);
#pragma unroll
    for (int off = GPW; off < kWave; off <<= 1) mx = fmaxf(mx, __shfl_xor(mx, off, kWave));
    const float mx_safe = (mx == -INFINITY) ? 0.f : mx;
    float lt = 0.f;
#pragma unroll
    for (int j = 0; j < EPL; ++j) lt = fmaf(el[j], fast_exp2(em[j] - mx_safe), lt);
#pragma unroll
    for (int off = GPW; off < kWave; off <<= 1) lt += __shfl_xor(lt, off, kWave);
    // lane g of the wavefront holds head g's maximum and denominator
    const float my_mx = __shfl(mx, g, kWave), my_l = __shfl(lt, g, kWave);
    const float m_safe = (my_mx == -INFINITY) ? 0.f : my_mx;

    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int s0 = 0; s0 < S; s0 += NS * KMAX) {
        if (s0 != 0) load_pass(s0);
#pragma unroll
        for (int k = 0; k < KMAX; ++k) {
            const int s = s0 + sg + NS * k;
            const float wgt = (worker && s < S) ? fast_exp2(xm[k] - m_safe) : 0.f;
            acc.x = fmaf(x[k].x, wgt, acc.x);
            acc.y = fmaf(x[k].y, wgt, acc.y);
            acc.z = fmaf(x[k].z, wgt, acc.z);
            acc.w = fmaf(x[k].w, wgt, acc.w);
        }
    }
    if (worker) *reinterpret_cast<float4 *>(s_red + (sg * COMBOS + rem) * 4) = acc;
    __syncthreads();
    if (tid < COMBOS) {
        float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int r = 0; r < NS; ++r) {
            const float4 t = *reinterpret_cast<const float4 *>(s_red + (r * COMBOS + rem) * 4);
            a.x += t.x; a.y += t.y; a.z += t.z; a.w += t.w;
        }
        const float l = my_l;
        const float inv = (l > 0.f) ? 1.0f / l : 0.f;
        const float o0 = a.x * inv, o1 = a.y * inv, o2 = a.z * inv, o3 = a.w * inv;
        const int64_t ooff = ((int64_t)b * p.Hq + (int64_t)h * G + g) * D + 4 * q4;
        if (p.o_is_bf16) {
            *reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(p.O) + ooff) = make_uint2(pack_bf16x2(o0, o1), pack_bf16x2(o2, o3));
        } else {
            *reinterpret_cast<float4 *>(reinterpret_cast<float *>(p.O) + ooff) = make_float4(o0, o1, o2, o3);
        }
        if (q4 == 0 && p.lse)
            p.lse[(int64_t)b * p.Hq + (int64_t)h * G + g] = (l > 0.f) ? (my_mx + __log2f(l)) * kLn2 : -INFINITY;
    }
}

template <int G> struct FastShape {
    static constexpr int WAVES = 6;                   // two such workgroups per CU: 12 waves x 8 KB of loads in flight, <= 170 VGPRs each
                                                      // (one workgroup of 12 waves per CU was 1-8 % slower on every configuration)
    static constexpr int THREADS = WAVES * kWave;
    static constexpr int U = 4;                       // wave-wide loads of K (and of V) per step: 16 rows, one MFMA tile
};

// TAIL: the rows of a (sequence, KV head) are its merged rows followed by the first tail_lens[b] rows of
// the uncompressed tail; a tail row is a cluster of one (bias ln 1 = 0).
template <int D, int G, bool TAIL>
__global__ __launch_bounds__(FastShape<G>::THREADS) void decode_bf16_kernel(DecParams p) {
    static_assert(D == 128, "16 lanes per row");
    constexpr int LPR = 16;
    constexpr int RPW = kWave / LPR;                       // 4 rows per wave-wide load
    static_assert(G >= 1 && G <= 16, "the query heads of a group are the 16 columns of one matrix tile");
    constexpr int WAVES = FastShape<G>::WAVES;
    constexpr int THREADS = FastShape<G>::THREADS;
    constexpr int U = FastShape<G>::U;
    static_assert(U == 4, "one step is one 16-row tile");
    constexpr int kRowsPerWaveStep = RPW * U;
    constexpr int kRowsPerBlockStep = kRowsPerWaveStep * WAVES;
    constexpr int kStride = D + kPartPad;   // floats per (split, head) partial: acc[D], m, l, pad
    constexpr int kBufFloats = (WAVES * G * D) > (THREADS * 4) ? (WAVES * G * D) : (THREADS * 4);

    // s_buf: per-wave accumulators [WAVES][G][D] first, the split-group sums of the final fold later
    __shared__ __attribute__((aligned(16))) float s_buf[kBufFloats];
    __shared__ float s_m[WAVES][G];
    __shared__ float s_l[WAVES][G];
    __shared__ int s_last;
    // per wave: 16 rows of keys turned around for the matrix cores
    constexpr int kKtRowBytes = 2 * D + 16;
    constexpr int kKtBytes = 16 * kKtRowBytes;
    __shared__ __attribute__((aligned(16))) char s_kt[WAVES * kKtBytes];

    // workgroup id = split * (B * Hkv) + (sequence, head): see publish_or_collect
    const int n_bh = p.B * p.Hkv;
    const int split = (int)blockIdx.x / n_bh;
    const int bh_i = (int)blockIdx.x - split * n_bh;
    const int b = bh_i / p.Hkv, h = bh_i - b * p.Hkv;
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);   // scalar: keeps the row loop wave-uniform
    const int g = lane / LPR, c = lane % LPR;
    const int64_t bh = bh_i;
    HeadSync *hs = p.sync + bh;
    const unsigned long long epoch = __hip_atomic_load(&hs->epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int rows_c = min(max(p.comp_lens[bh], 0), p.cap);
    const int rows_total = rows_c + (TAIL ? min(max(p.tail_lens[b], 0), p.tail_cap) : 0);
    const int S = splits_for(rows_total, p.max_splits, p.min_rows);
    if (split >= S) return;
    if (epoch == kEpochPoison) {   // an earlier call on this workspace failed: fail again, visibly
        if (split == S - 1) file_failure<G, D>(p, hs, b, h, tid, THREADS);
        return;
    }
    const bool local = p.local != 0;
    // contiguous row range of this split, a multiple of the block step except for the last one
    int per = (rows_total + S - 1) / S;
    per = (per + kRowsPerBlockStep - 1) / kRowsPerBlockStep * kRowsPerBlockStep;
    const int r0 = min(split * per, rows_total), r1 = min(r0 + per, rows_total);

    // Rows come through buffer descriptors that end at this split's last row: the hardware returns zeros for
    // anything beyond, so no load needs a predicate, a branch or a 64-bit address (the launcher checks that
    // the byte offsets of a (sequence, head) fit in 31 bits).  A row of zeros with size 0 is "no row".
    const int end_c = min(r1, rows_c);                       // merged rows of this split end here
    const int end_t = TAIL ? max(r1 - rows_c, 0) : 0;        // tail rows of this split end here
    const auto k_src = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(reinterpret_cast<const bf16_t *>(p.Kc) + bh * (int64_t)p.cap * D),
                                                         (short)0, end_c * D * 2, 0x00020000);
    const auto v_src = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(reinterpret_cast<const bf16_t *>(p.Vc) + bh * (int64_t)p.cap * D),
                                                         (short)0, end_c * D * 2, 0x00020000);
    const auto n_src = __builtin_amdgcn_make_buffer_rsrc(const_cast<int32_t *>(p.counts + bh * (int64_t)p.cap), (short)0, end_c * 4, 0x00020000);
    const auto kt_src = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(reinterpret_cast<const bf16_t *>(TAIL ? p.Kt : p.Kc) + (TAIL ? bh * (int64_t)p.tail_cap * D : 0)),
                                                          (short)0, end_t * D * 2, 0x00020000);
    const auto vt_src = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(reinterpret_cast<const bf16_t *>(TAIL ? p.Vt : p.Vc) + (TAIL ? bh * (int64_t)p.tail_cap * D : 0)),
                                                          (short)0, end_t * D * 2, 0x00020000);

    uint4 kb[U], vb[U];
    int cb[U];
    // keys first, then sizes, then values: the scores are formed while the values are still on their way.
    // WHERE: 0 = the 16 rows of the step are merged rows, 1 = all of them are tail rows, 2 = the one step per
    // (sequence, head) that holds the last merged and the first tail rows: only that one asks both sources.
    auto issue_from = [&](int base, auto where) {
        constexpr int WHERE = decltype(where)::value;
        const int row0 = base + g;
        const int off0 = row0 * (D * 2) + 16 * c;
        int toff[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            // a row before the tail must not turn into a small offset by wrapping around
            const int rel = row0 + u * RPW - rows_c;
            toff[u] = (rel >= 0) ? rel * (D * 2) + 16 * c : (int)0x80000000;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            dec_u32x4 v = {0u, 0u, 0u, 0u};
            if (WHERE != 1) v = __builtin_amdgcn_raw_buffer_load_b128(k_src, off0 + u * RPW * D * 2, 0, kAuxStream);
            if (WHERE == 1) v = __builtin_amdgcn_raw_buffer_load_b128(kt_src, toff[u], 0, kAuxStream);
            if (WHERE == 2) v |= __builtin_amdgcn_raw_buffer_load_b128(kt_src, toff[u], 0, kAuxStream);
            kb[u] = make_uint4(v.x, v.y, v.z, v.w);
        }
        __builtin_amdgcn_sched_barrier(0);     // keep the order of the requests: the scheduler has no reason to
#pragma unroll
        for (int u = 0; u < U; ++u) {
            cb[u] = (WHERE != 1) ? (int)__builtin_amdgcn_raw_buffer_load_b32(n_src, (row0 + u * RPW) * 4, 0, kAuxStream) : 0;
            if (WHERE != 0) cb[u] = (toff[u] >= 0 && row0 + u * RPW < r1) ? 1 : cb[u];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            dec_u32x4 v = {0u, 0u, 0u, 0u};
            if (WHERE != 1) v = __builtin_amdgcn_raw_buffer_load_b128(v_src, off0 + u * RPW * D * 2, 0, kAuxStream);
            if (WHERE == 1) v = __builtin_amdgcn_raw_buffer_load_b128(vt_src, toff[u], 0, kAuxStream);
            if (WHERE == 2) v |= __builtin_amdgcn_raw_buffer_load_b128(vt_src, toff[u], 0, kAuxStream);
            vb[u] = make_uint4(v.x, v.y, v.z, v.w);
        }
    };
    auto issue = [&](int base) {      // (base and rows_c are the same for the whole wavefront)
        if (!TAIL || base + kRowsPerWaveStep <= rows_c) issue_from(base, std::integral_constant<int, 0>{});
        else if (base >= rows_c) issue_from(base, std::integral_constant<int, 1>{});
        else issue_from(base, std::integral_constant<int, 2>{});
    };
    int base = r0 + wave * kRowsPerWaveStep;
    issue(base);

    float m_run = -INFINITY, l_run = 0.f;
    {
        // Both products on the matrix cores, 16 rows per step (v_mfma_f32_16x16x32_bf16 for the scores, whose
        // contraction runs over the 128 elements of a row; v_mfma_f32_16x16x16_bf16 for the sums, whose
        // contraction is the 16 rows of the step).
        //   S = K_c q^T: the rows are spread over the lanes by column (16-byte pieces), the A operand wants
        //   one row per lane position, so the wave turns its 16 rows around through a 4 KB tile in LDS
        //   (row stride 272 B: the operand reads are free of bank conflicts).  Register u of lane group g
        //   is row 4u + g and goes to tile row 4g + u; B holds the query heads (lane position c = head c,
        //   zero beyond the group).  The result leaves lane (g, c) with the scores of head c for tile
        //   rows 4g + i = rows 4i + g, i = 0..3: the rows whose sizes the lane group loaded itself.
        //   O += P V: the 16 rows are the contraction index, A[m][k] = probability of head m for row k, and
        //   the k index (lane / 16, i) of both operands stands for row 4i + lane / 16: the probabilities
        //   are used where the first product left them, and B[k][n] = element 8c + j of row k is built
        //   from the loaded registers with two byte permutes per product, one product per j.
        // The second product adds up the rows of all four lane groups: they share one running maximum per
        // head, and the result holds the whole wave's sums: accm[j][i] of lane (g, c) = head 4g + i, element
        // 8c + j (for groups of up to four heads only lanes 0..15 hold anything).
        // P enters as two bf16 parts (leading part and remainder), so its rounding error is 2^-18.
        char *kt = s_kt + wave * kKtBytes;
        // B operand of the first product: lane (g, c) holds elements 32ks + 8g .. + 7 of head c (zeros for c >= G:
        // the descriptor ends after the G heads of the group)
        uint4 qb[4];
        {
            const auto q_src = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(reinterpret_cast<const bf16_t *>(p.Q) + ((int64_t)b * p.Hq + (int64_t)h * G) * D),
                                                                 (short)0, G * D * 2, 0x00020000);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const dec_u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(q_src, c * (D * 2) + (32 * ks + 8 * g) * 2, 0, 0);
                qb[ks] = make_uint4(v.x, v.y, v.z, v.w);
            }
        }
        f32x4_t accm[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) accm[j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        while (base < r1) {
#pragma unroll
            for (int u = 0; u < U; ++u) *reinterpret_cast<uint4 *>(kt + (4 * g + u) * kKtRowBytes + 16 * c) = kb[u];
            wave_lds_handover();
            f32x4_t sc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const uint4 a = *reinterpret_cast<const uint4 *>(kt + c * kKtRowBytes + (32 * ks + 8 * g) * 2);
                sc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(dec_bf16x8, a),
                                                             __builtin_bit_cast(dec_bf16x8, qb[ks]), sc, 0, 0, 0);
            }
            wave_lds_handover();     // the tile is rewritten in the next step
            float sv[4];
            float m_loc = m_run;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                sv[i] = (cb[i] > 0) ? fmaf(sc[i], p.scale_log2, __log2f((float)cb[i])) : -INFINITY;
                m_loc = fmaxf(m_loc, sv[i]);
            }
            const float m_new = rows_allreduce_max(m_loc);
            const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
            const float alpha = fast_exp2(m_run - m_safe);
            float pi[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) pi[i] = fast_exp2(sv[i] - m_safe);
            l_run = fmaf(l_run, alpha, (pi[0] + pi[1]) + (pi[2] + pi[3]));   // per lane group; added up after the loop
            m_run = m_new;
            if (ballot64(alpha != 1.0f) != 0ull) {
                // the factor of head 4g + i sits at lane position 4g + i of every 16-lane row
                float al[4];
                if constexpr (G <= 4) {
                    BcastAll<4>::run(alpha, al);
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i) al[i] = lane_gather(alpha, 20 * g + i);
                }
#pragma unroll
                for (int j = 0; j < 8; ++j)
#pragma unroll
                    for (int i = 0; i < 4; ++i) accm[j][i] *= al[i];
            }
            const uint32_t h01 = pack_bf16x2(pi[0], pi[1]), h23 = pack_bf16x2(pi[2], pi[3]);
            const uint32_t r01 = pack_bf16x2(pi[0] - bf16_lo(h01), pi[1] - bf16_hi(h01));
            const uint32_t r23 = pack_bf16x2(pi[2] - bf16_lo(h23), pi[3] - bf16_hi(h23));
            const dec_short4 a_hi = __builtin_bit_cast(dec_short4, make_uint2(h01, h23));
            const dec_short4 a_lo = __builtin_bit_cast(dec_short4, make_uint2(r01, r23));
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint32_t d0 = dword_of(vb[0], j >> 1), d1 = dword_of(vb[1], j >> 1);
                const uint32_t d2 = dword_of(vb[2], j >> 1), d3 = dword_of(vb[3], j >> 1);
                const uint32_t lo = (j & 1) ? pack_hi(d0, d1) : pack_lo(d0, d1);
                const uint32_t hi = (j & 1) ? pack_hi(d2, d3) : pack_lo(d2, d3);
                const dec_short4 bb = __builtin_bit_cast(dec_short4, make_uint2(lo, hi));
                accm[j] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a_hi, bb, accm[j], 0, 0, 0);
                accm[j] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a_lo, bb, accm[j], 0, 0, 0);
            }
            base += kRowsPerBlockStep;
            if (base < r1) issue(base);
        }
        // ---- park the wave's sums in LDS (m_run is already the same in all lane groups)
        const float lw = rows_allreduce_sum(l_run);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int hh = 4 * g + i;
            if (hh < G) {
                float *dst = s_buf + (wave * G + hh) * D + 8 * c;
                *reinterpret_cast<float4 *>(dst) = make_float4(accm[0][i], accm[1][i], accm[2][i], accm[3][i]);
                *reinterpret_cast<float4 *>(dst + 4) = make_float4(accm[4][i], accm[5][i], accm[6][i], accm[7][i]);
            }
        }
        if (g == 0 && c < G) { s_m[wave][c] = m_run; s_l[wave][c] = lw; }
    }
    __syncthreads();
    // ---- fold the waves, write this split's partial
    float *part_bh = p.part + bh * (int64_t)p.max_splits * G * kStride;
    for (int i = tid; i < G * D; i += THREADS) {
        const int hh = i / D, e = i % D;
        float mw = -INFINITY;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) mw = fmaxf(mw, s_m[w][hh]);
        const float m_safe = (mw == -INFINITY) ? 0.f : mw;
        float a = 0.f, l = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) {
            const float f = fast_exp2(s_m[w][hh] - m_safe);
            a = fmaf(s_buf[(w * G + hh) * D + e], f, a);
            l = fmaf(s_l[w][hh], f, l);
        }
        float *dst = part_bh + ((int64_t)split * G + hh) * kStride;
        store_partial(dst + e, a, local);
        if (e == 0) { store_partial(dst + D, mw, local); store_partial(dst + D + 1, l, local); }
    }
    // ---- the workgroup of the last split folds all splits
    const int got = publish_or_collect(hs, epoch, S, split, tid, local, p.poll_budget, &s_last);
    if (got == 0) return;
    if (got < 0) {
        file_failure<G, D>(p, hs, b, h, tid, THREADS);
        return;
    }
    combine_splits<D, G, THREADS>(p, part_bh, S, b, h, tid, s_buf);
    if (tid == 0) __hip_atomic_store(&hs->epoch, epoch + 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ------------------------------------------------------------------------------------------------
// Generic kernel: every lane group reduces with a DPP all-reduce and updates the softmax state of all
// G heads itself; the last workgroup folds the partials one (head, element) per thread.
template <typename T, int D, int G>
__global__ __launch_bounds__(kDecThreads) void decode_generic_kernel(DecParams p) {
    constexpr int LPR = D / 8;
    constexpr int RPW = kWave / LPR;
    constexpr int kRowsPerWaveStep = RPW * kDecUnroll;
    constexpr int kRowsPerBlockStep = kRowsPerWaveStep * kDecWaves;
    constexpr int kStride = D + kPartPad;   // floats per (split, head) partial: acc[D], m, l, pad

    __shared__ float s_acc[kDecWaves][G][D];
    __shared__ float s_m[kDecWaves][G];
    __shared__ float s_l[kDecWaves][G];
    __shared__ __attribute__((aligned(16))) float s_red[kDecThreads * 4];
    __shared__ int s_last;

    // workgroup id = split * (B * Hkv) + (sequence, head): see publish_or_collect
    const int n_bh = p.B * p.Hkv;
    const int split = (int)blockIdx.x / n_bh;
    const int bh_i = (int)blockIdx.x - split * n_bh;
    const int b = bh_i / p.Hkv, h = bh_i - b * p.Hkv;
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);   // scalar: keeps the row loop wave-uniform
    const int g = lane / LPR, c = lane % LPR;
    const int64_t bh = bh_i;
    HeadSync *hs = p.sync + bh;
    const unsigned long long epoch = __hip_atomic_load(&hs->epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int rows_c = min(max(p.comp_lens[bh], 0), p.cap);
    // merged rows, then the uncompressed tail (if the call has one): a tail row is a cluster of one
    const int rows_total = rows_c + (p.Kt ? min(max(p.tail_lens[b], 0), p.tail_cap) : 0);
    const int S = splits_for(rows_total, p.max_splits, p.min_rows);
    if (split >= S) return;
    if (epoch == kEpochPoison) {   // an earlier call on this workspace failed: fail again, visibly
        if (split == S - 1) file_failure<G, D>(p, hs, b, h, tid, kDecThreads);
        return;
    }
    const bool local = p.local != 0;
    // contiguous row range of this split, a multiple of the block step except for the last one
    int per = (rows_total + S - 1) / S;
    per = (per + kRowsPerBlockStep - 1) / kRowsPerBlockStep * kRowsPerBlockStep;
    const int r0 = min(split * per, rows_total), r1 = min(r0 + per, rows_total);

    const T *Kbh = reinterpret_cast<const T *>(p.Kc) + bh * (int64_t)p.cap * D;
    const T *Vbh = reinterpret_cast<const T *>(p.Vc) + bh * (int64_t)p.cap * D;
    const int32_t *cnt_bh = p.counts + bh * (int64_t)p.cap;
    const T *Ktbh = reinterpret_cast<const T *>(p.Kt) + bh * (int64_t)p.tail_cap * D;
    const T *Vtbh = reinterpret_cast<const T *>(p.Vt) + bh * (int64_t)p.tail_cap * D;

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
            if (ok[u] && row >= rows_c) {
                load8(Ktbh + (int64_t)(row - rows_c) * D + 8 * c, kk[u]);
                load8(Vtbh + (int64_t)(row - rows_c) * D + 8 * c, vv[u]);
                bias[u] = 0.f;
            } else if (ok[u]) {
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
        store_partial(dst + e, a, local);
        if (e == 0) { store_partial(dst + D, mw, local); store_partial(dst + D + 1, l, local); }
    }

    // ---- the workgroup of the last split folds all splits
    const int got = publish_or_collect(hs, epoch, S, split, tid, local, p.poll_budget, &s_last);
    if (got == 0) return;
    if (got < 0) {
        file_failure<G, D>(p, hs, b, h, tid, kDecThreads);
        return;
    }
    combine_splits<D, G, kDecThreads>(p, part_bh, S, b, h, tid, s_red);
    if (tid == 0) __hip_atomic_store(&hs->epoch, epoch + 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__global__ void zero_words_kernel(int32_t *p, size_t n) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

size_t decode_workspace_state_bytes(int B, int Hkv) { return kDecStatusBytes + align_up((size_t)B * Hkv * sizeof(HeadSync), 256); }

static int clamp_splits() { return max(1, min(kDecMaxSplits, tuning().decode_max_splits)); }   // knob <= 0: automatic

size_t decode_workspace_bytes(int B, int Hq, int Hkv, int /* cap: the size does not depend on it */, int d) {
    const int G = Hq / Hkv;
    // sized for the largest split count the tuning knob may take, so the knob never invalidates a workspace
    const size_t split_k = align_up((size_t)B * Hkv * kDecMaxSplits * G * (d + kPartPad) * 4, 256);
    // (see launch_decode; sized for any number of rows, the tail's capacity is not known here)
    const size_t mfma = (d == 128) ? multi_fast_workspace_bytes(B, Hq, Hkv, 1, 1 << 30) : 0;
    return decode_workspace_state_bytes(B, Hkv) + (split_k > mfma ? split_k : mfma);
}

// ------------------------------------------------------------------------------------------------
// Scratch of sc_decode_attn_static: one file-scope array per GPU, for callers that cannot hand in a
// workspace because they cannot allocate one.  Its name is only a host-side stand-in; the device
// address is looked up once per device and only that pointer is ever given to a kernel.  The array is
// zero when the code object is loaded, which is the state the flags at its start must have, and
// every call leaves them zero again.
static __device__ __align__(256) unsigned char scratch[kDecodeStaticArrayBytes];
static_assert(kDecodeStaticStateBytes == kDecStatusBytes + kDecodeStaticMaxHeads * sizeof(HeadSync) && kDecodeStaticStateBytes % 256 == 0,
              "state region of the static scratch");

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void *g_scratch_ptr[kMaxDevices] = {};

hipError_t decode_static_scratch(void **ptr) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return hipSuccess;
}

hipError_t launch_decode_init_workspace(void *ws, size_t state_bytes, hipStream_t stream) {
    const size_t n = state_bytes / 4;
    hipLaunchKernelGGL(zero_words_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream,
                       reinterpret_cast<int32_t *>(ws), n);
    return hipGetLastError();
}

template <typename T, int D, int G>
static hipError_t launch_g(const DecParams &p, hipStream_t stream) {
    const dim3 grid((unsigned)p.max_splits * (unsigned)(p.Hkv * p.B));
    if constexpr (D == 128 && sizeof(T) == 2) {
        // the fast kernel addresses the rows of a (sequence, head) with 32-bit byte offsets
        const int64_t reach = ((int64_t)(p.cap > p.tail_cap ? p.cap : p.tail_cap) + 2 * FastShape<G>::THREADS) * D * 2;
        if (p.q_is_bf16 && reach < (1ll << 31)) {
            if (p.Kt) hipLaunchKernelGGL((decode_bf16_kernel<D, G, true>), grid, dim3(FastShape<G>::THREADS), 0, stream, p);
            else hipLaunchKernelGGL((decode_bf16_kernel<D, G, false>), grid, dim3(FastShape<G>::THREADS), 0, stream, p);
            return hipGetLastError();
        }
    }
    hipLaunchKernelGGL((decode_generic_kernel<T, D, G>), grid, dim3(kDecThreads), 0, stream, p);
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
    // Optional route (knob, off by default): a single query row through the kernel for blocks of query rows,
    // which treats the G heads as one 16-row tile, writes partials and folds them in a second launch.  The
    // decode kernel above measured level or slightly ahead of it for every group size (35.3 against 36.1 us
    // at G = 7 on a ragged batch of 32).  Its partials go behind the flags, which it neither needs nor touches.
    if (a.kv_dtype == DType::BF16 && a.q_dtype == DType::BF16 && a.d == 128 &&
        a.Hq / a.Hkv >= tuning().decode_mfma_min_group) {
        MultiArgs m;
        m.Q = a.Q; m.q_dtype = a.q_dtype; m.nq = 1;
        m.Kc = a.Kc; m.Vc = a.Vc; m.kv_dtype = a.kv_dtype; m.cap = a.cap;
        m.counts = a.counts; m.comp_lens = a.comp_lens;
        m.Kt = a.Kt; m.Vt = a.Vt; m.tail_lens = a.tail_lens; m.tail_cap = a.tail_cap;
        m.B = a.B; m.Hq = a.Hq; m.Hkv = a.Hkv; m.d = a.d;
        m.scale = a.scale;
        m.O = a.O; m.o_dtype = a.o_dtype; m.lse = a.lse;
        m.ws = reinterpret_cast<char *>(a.ws) + (a.state_bytes ? a.state_bytes : decode_workspace_state_bytes(a.B, a.Hkv));
        return launch_multi_fast(m, stream);
    }
    DecParams p;
    p.Q = a.Q; p.q_is_bf16 = a.q_dtype == DType::BF16;
    p.Kc = a.Kc; p.Vc = a.Vc; p.cap = a.cap;
    p.counts = a.counts; p.comp_lens = a.comp_lens;
    p.Kt = a.Kt; p.Vt = a.Vt; p.tail_lens = a.tail_lens; p.tail_cap = a.Kt ? a.tail_cap : 0;
    p.B = a.B; p.Hq = a.Hq; p.Hkv = a.Hkv;
    p.scale_log2 = a.scale * kLog2e;
    p.O = a.O; p.o_is_bf16 = a.o_dtype == DType::BF16;
    p.lse = a.lse;
    p.status = reinterpret_cast<int32_t *>(a.ws);
    p.sync = reinterpret_cast<HeadSync *>(reinterpret_cast<char *>(a.ws) + kDecStatusBytes);
    p.part = reinterpret_cast<float *>(reinterpret_cast<char *>(a.ws) +
                                       (a.state_bytes ? a.state_bytes : decode_workspace_state_bytes(a.B, a.Hkv)));
    // the hardware hands consecutive workgroup ids to the 8 XCCs in turn: with B * Hkv a multiple of 8 the id
    // (split * B * Hkv + head) keeps every head on one XCC
    p.local = ((a.B * a.Hkv) % 8 == 0 && tuning().decode_local_handover) ? 1 : 0;
    p.poll_budget = tuning().decode_poll_budget;
    p.min_rows = max(1, tuning().decode_min_rows);
    // Splits per (sequence, KV head): enough workgroups to cover the 256 CUs about once; more splits
    // only add partials to fold and tickets to take (both are serial tails of the kernel).
    int splits = clamp_splits();
    if (tuning().decode_max_splits <= 0) splits = max(2, min(32, 256 / max(1, a.B * a.Hkv)));
    // never more splits than the capacity can feed
    const int by_cap = (a.cap + p.tail_cap + p.min_rows - 1) / p.min_rows;
    p.max_splits = max(1, min(splits, by_cap));
    const int G = a.Hq / a.Hkv;
    if (a.kv_dtype == DType::BF16)
        return a.d == 128 ? launch_td<bf16_t, 128>(p, G, stream) : launch_td<bf16_t, 64>(p, G, stream);
    return a.d == 128 ? launch_td<float, 128>(p, G, stream) : launch_td<float, 64>(p, G, stream);
}

}  // namespace sc
