// sc_multi_attn: Proportional Attention for a block of query rows (paper Sec. 2.4, Eq. 4 with
// Q in R^{n x d}):   O[j] = softmax(Q[j] K_c^T * scale + ln s) V_c   for every query row j, no mask.
//
// Fast path (bf16 queries and cache, d = 128) on the matrix cores.  The query rows that share a KV head
// -- (query j, head g of the group), nq * G of them -- are cut into blocks of 32 = two MFMA tiles; a
// workgroup of four wavefronts owns one block and one contiguous range of cache rows (split-K), its
// wavefronts take alternate 32-row steps of that range.  Per step and wavefront:
//   * S^T = K_c Q^T with v_mfma_f32_16x16x32_bf16: the cache rows are the A operand, the query rows the
//     B operand, both loaded straight from memory in operand layout (lane l: row l%16, 16-byte piece
//     l/16 + 4j of the row; the contraction index may be permuted freely as long as both sides agree).
//     The result lands with the query row on l%16 and four cache rows per lane, which is exactly the A
//     layout of the second product, so the probabilities never move between lanes.
//   * scale, + log2(size) bias, online softmax per query row (exp2 domain): in-lane over the lane's
//     cache rows, then over the four lane groups with two row swaps.
//   * O += P V with the same MFMA (the 32 rows of a step are one contraction); P enters as two bf16 parts
//     (leading part + remainder, two products), V rows loaded 16 bytes per lane and regrouped with v_perm
//     into the B operand (column 8c + j on lane c).
// The four wavefronts fold through LDS, the workgroup writes one partial (acc[128], m, l) per query
// row, and a second small kernel folds the splits.  Two launches instead of a hand-over inside the
// kernel: the call is for several rows at once, a few microseconds of launch matter less than for
// single-row decode.
//
// Everything else (fp32, d = 64) goes row by row through the decode kernels.
#include "sc_device.h"
#include "sc_host.h"

namespace sc {

typedef float mq_float4 __attribute__((ext_vector_type(4)));

constexpr int kMqD = 128;
constexpr int kMqRows = 32;                       // query rows per workgroup at most (two MFMA tiles)
constexpr int kMqWaves = 4;
constexpr int kMqThreads = kMqWaves * kWave;
constexpr int kMqStep = 32;                       // cache rows per wavefront and softmax update
constexpr int kMqBlockStep = kMqStep * kMqWaves;
constexpr int kMqMaxSplits = 64;
constexpr int kMqPart = kMqD + 4;                 // floats per partial row: acc[128], m, l, pad
constexpr float kMqLog2e = 1.4426950408889634f;
constexpr float kMqLn2 = 0.6931471805599453f;

struct MqParams {
    const bf16_t *Q;          // [nq, B, Hq, 128]
    const bf16_t *Kc, *Vc;    // [B, Hkv, cap, 128]
    const int32_t *counts, *comp_lens;
    const bf16_t *Kt, *Vt;    // uncompressed tail [B, Hkv, tail_cap, 128], or NULL
    const int32_t *tail_lens; // [B]
    int tail_cap, causal;     // causal: the last nq tail rows are the query rows' own tokens
    int nq, cap, B, Hq, Hkv, G;
    float scale_log2;
    float *part;              // [B*Hkv*row_blocks][max_splits][32][kMqPart]
    int row_blocks, max_splits, min_rows;
    int block_rows;           // query rows per workgroup: 16 (one MFMA tile) when nq * G <= 16, else 32
    void *O;                  // [nq, B, Hq, 128]
    int o_is_bf16;
    float *lse;               // [nq, B, Hq] or NULL
};

__device__ __forceinline__ int mq_splits_for(int rows, int max_splits, int min_rows) {
    const int s = (rows + min_rows - 1) / min_rows;
    return s < 1 ? 1 : (s > max_splits ? max_splits : s);
}
typedef __bf16 mq_bf16x8 __attribute__((ext_vector_type(8)));
__device__ __forceinline__ mq_bf16x8 mq_op8(const uint4 &u) { return __builtin_bit_cast(mq_bf16x8, u); }
// max / sum over the four 16-lane rows of a wavefront, same position in the row
__device__ __forceinline__ float mq_rows_max(float x) {
    auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
    r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float mq_rows_sum(float x) {
    auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float mq_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// QT: MFMA tiles of query rows per workgroup (1 or 2).  TAIL: the rows of a (sequence, KV head) are its
// merged rows followed by the first tail_lens[b] rows of the tail (size 1); with `causal` query j sees the
// tail rows up to its own token, tail_lens[b] - nq + j.
template <int QT, bool TAIL>
__global__ __launch_bounds__(kMqThreads, QT == 1 ? 2 : 1) void multi_attn_kernel(MqParams p) {
    constexpr int kRows = 16 * QT;
    __shared__ __attribute__((aligned(16))) float s_acc[kRows * kMqD];
    __shared__ float s_m[kMqWaves][kRows];
    __shared__ float s_l[kMqWaves][kRows];

    const int split = blockIdx.x;
    const int rb = (int)blockIdx.y / p.Hkv, h = (int)blockIdx.y - rb * p.Hkv;
    const int b = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int c = lane & 15, kq = lane >> 4;
    const int64_t bh = (int64_t)b * p.Hkv + h;
    // (made scalar explicitly: the row loop below holds wave-wide operations and must not diverge)
    const int rows_c = __builtin_amdgcn_readfirstlane(min(max(p.comp_lens[bh], 0), p.cap));
    const int rows_t = TAIL ? __builtin_amdgcn_readfirstlane(min(max(p.tail_lens[b], 0), p.tail_cap)) : 0;
    const int rows_total = rows_c + rows_t;
    const int S = mq_splits_for(rows_total, p.max_splits, p.min_rows);
    if (split >= S) return;
    int per = (rows_total + S - 1) / S;
    per = (per + kMqBlockStep - 1) / kMqBlockStep * kMqBlockStep;
    const int r0 = min(split * per, rows_total), r1 = min(r0 + per, rows_total);

    const bf16_t *Kbh = p.Kc + bh * (int64_t)p.cap * kMqD;
    const bf16_t *Vbh = p.Vc + bh * (int64_t)p.cap * kMqD;
    const int32_t *cnt_bh = p.counts + bh * (int64_t)p.cap;
    const bf16_t *Ktbh = TAIL ? p.Kt + bh * (int64_t)p.tail_cap * kMqD : nullptr;
    const bf16_t *Vtbh = TAIL ? p.Vt + bh * (int64_t)p.tail_cap * kMqD : nullptr;

    // query rows of the block as B operands: lane (c, kq) holds pieces kq, kq + 4, kq + 8, kq + 12 of row c
    uint4 qop[QT][4];
    int limit[QT];                             // rows [0, limit) are visible to query row (qt, c)
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        const int R = rb * kRows + qt * 16 + c;
        const bool valid = R < p.nq * p.G;
        const int j = valid ? R / p.G : 0;
        const int g = valid ? R - j * p.G : 0;
        const bf16_t *qp = p.Q + (((int64_t)j * p.B + b) * p.Hq + (int64_t)h * p.G + g) * kMqD;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj)
            qop[qt][jj] = valid ? *reinterpret_cast<const uint4 *>(qp + 8 * (kq + 4 * jj)) : make_uint4(0, 0, 0, 0);
        limit[qt] = rows_c + ((TAIL && p.causal) ? max(0, rows_t - p.nq + 1 + j) : rows_t);
    }

    float m_run[QT];   // per query row (qt, c), identical on the four lane groups
    float l_run[QT];               // this lane's share (its cache rows) of the row's sum
    mq_float4 o[QT][8];                         // o[qt][jn][i]: query row qt*16 + 4kq + i, column 8c + jn
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        m_run[qt] = -INFINITY;
        l_run[qt] = 0.f;
#pragma unroll
        for (int jn = 0; jn < 8; ++jn) o[qt][jn] = mq_float4{0.f, 0.f, 0.f, 0.f};
    }

    // one step of loads: the keys of 32 cache rows in operand layout, their values 16 bytes per lane, sizes
    struct StepRegs {
        uint4 kop[2][4], vr[2][4];
        int cnt[2][4];
    };
    // With one block of query rows every cache row is read once by the launch: the loads carry the
    // non-temporal hint.  Several row blocks read the cache again, from the caches: no hint then.
    auto get16 = [&](const bf16_t *ptr) {
        return (p.row_blocks == 1) ? load16_stream(ptr) : *reinterpret_cast<const uint4 *>(ptr);
    };
    auto load_step = [&](int base, StepRegs &x) {
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int row0 = base + 16 * t;
            const int krow = row0 + c;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj)
                x.kop[t][jj] = (krow >= r1) ? make_uint4(0, 0, 0, 0)
                               : (TAIL && krow >= rows_c) ? get16(Ktbh + (int64_t)(krow - rows_c) * kMqD + 8 * (kq + 4 * jj))
                                                          : get16(Kbh + (int64_t)krow * kMqD + 8 * (kq + 4 * jj));
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int vrow = row0 + 4 * kq + i;
                if (vrow >= r1) {
                    x.vr[t][i] = make_uint4(0, 0, 0, 0);
                    x.cnt[t][i] = 0;
                } else if (TAIL && vrow >= rows_c) {
                    x.vr[t][i] = get16(Vtbh + (int64_t)(vrow - rows_c) * kMqD + 8 * c);
                    x.cnt[t][i] = 1;
                } else {
                    x.vr[t][i] = get16(Vbh + (int64_t)vrow * kMqD + 8 * c);
                    x.cnt[t][i] = cnt_bh[vrow];
                }
            }
        }
    };
    auto compute_step = [&](const StepRegs &x, int base) {
        const auto &kop = x.kop;
        const auto &vr = x.vr;
        const auto &cnt = x.cnt;
        // ---- logits: z[t][qt][i] for cache row base + 16t + 4kq + i and query row qt*16 + c
        float z[2][QT][4];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int qt = 0; qt < QT; ++qt) {
                mq_float4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int jj = 0; jj < 4; ++jj)     // a 16-byte piece per lane is one 32-element slice of the contraction
                    s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(mq_op8(kop[t][jj]), mq_op8(qop[qt][jj]), s, 0, 0, 0);
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    z[t][qt][i] = (cnt[t][i] > 0 && (!TAIL || base + 16 * t + 4 * kq + i < limit[qt]))
                                      ? fmaf(s[i], p.scale_log2, __log2f((float)cnt[t][i])) : -INFINITY;
            }
        // ---- online softmax per query row
        // probabilities as bf16: leading part and remainder; a lane's eight cache rows (4 of each half step) are
        // its share of the 32-row contraction of the second product
        uint4 pa[QT], pb[QT];
        float alpha[QT];
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) {
            float mx = -INFINITY;
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int i = 0; i < 4; ++i) mx = fmaxf(mx, z[t][qt][i]);
            mx = mq_rows_max(mx);
            const float m_new = fmaxf(m_run[qt], mx);
            const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
            alpha[qt] = mq_exp2(m_run[qt] - m_safe);
            m_run[qt] = m_new;
            float psum = 0.f;
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                // p = hi + lo with both parts bf16: two products instead of one keep 16 bits of every weight
                const float e0 = mq_exp2(z[t][qt][0] - m_safe), e1 = mq_exp2(z[t][qt][1] - m_safe);
                const float e2 = mq_exp2(z[t][qt][2] - m_safe), e3 = mq_exp2(z[t][qt][3] - m_safe);
                const uint32_t p01 = pack_bf16x2(e0, e1), p23 = pack_bf16x2(e2, e3);
                const uint32_t r01 = pack_bf16x2(e0 - bf16_lo(p01), e1 - bf16_hi(p01));
                const uint32_t r23 = pack_bf16x2(e2 - bf16_lo(p23), e3 - bf16_hi(p23));
                psum += (e0 + e1) + (e2 + e3);
                if (t == 0) { pa[qt].x = p01; pa[qt].y = p23; pb[qt].x = r01; pb[qt].y = r23; }
                else { pa[qt].z = p01; pa[qt].w = p23; pb[qt].z = r01; pb[qt].w = r23; }
            }
            l_run[qt] = fmaf(l_run[qt], alpha[qt], psum);
        }
        // ---- rescale the accumulators when a maximum moved (their rows are 4kq + i, the factors sit on lane row)
        bool moved = false;
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) moved = moved || (alpha[qt] != 1.0f);
        if (__ballot(moved) != 0ull) {
#pragma unroll
            for (int qt = 0; qt < QT; ++qt)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float a = __shfl(alpha[qt], 4 * kq + i, kWave);
#pragma unroll
                    for (int jn = 0; jn < 8; ++jn) o[qt][jn][i] *= a;
                }
        }
        // ---- O += P V
#pragma unroll
        for (int jn = 0; jn < 8; ++jn) {
            uint32_t w[4];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const uint32_t d0 = dword_of(vr[t][0], jn >> 1), d1 = dword_of(vr[t][1], jn >> 1);
                const uint32_t d2 = dword_of(vr[t][2], jn >> 1), d3 = dword_of(vr[t][3], jn >> 1);
                w[2 * t] = (jn & 1) ? pack_hi(d0, d1) : pack_lo(d0, d1);
                w[2 * t + 1] = (jn & 1) ? pack_hi(d2, d3) : pack_lo(d2, d3);
            }
            const mq_bf16x8 bb = mq_op8(make_uint4(w[0], w[1], w[2], w[3]));
#pragma unroll
            for (int qt = 0; qt < QT; ++qt) {
                o[qt][jn] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(mq_op8(pa[qt]), bb, o[qt][jn], 0, 0, 0);
                o[qt][jn] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(mq_op8(pb[qt]), bb, o[qt][jn], 0, 0, 0);
            }
        }
    };
    // two register sets: the loads of the next step fly while this one is computed
    {
        StepRegs xa, xb;
        int base = r0 + wave * kMqStep;
        if (base < r1) load_step(base, xa);
        while (base < r1) {
            const int next = base + kMqBlockStep;
            if (next < r1) load_step(next, xb);
            compute_step(xa, base);
            if (next >= r1) break;
            const int next2 = next + kMqBlockStep;
            if (next2 < r1) load_step(next2, xa);
            compute_step(xb, next);
            base = next2;
        }
    }

    // ---- fold the four wavefronts through LDS
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        const float lw = mq_rows_sum(l_run[qt]);
        if (kq == 0) { s_m[wave][qt * 16 + c] = m_run[qt]; s_l[wave][qt * 16 + c] = lw; }
    }
    __syncthreads();
    float f[QT][4];      // this wavefront's factor for query rows qt*16 + 4kq + i
#pragma unroll
    for (int qt = 0; qt < QT; ++qt)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = qt * 16 + 4 * kq + i;
            float mw = -INFINITY;
#pragma unroll
            for (int w = 0; w < kMqWaves; ++w) mw = fmaxf(mw, s_m[w][row]);
            const float m_safe = (mw == -INFINITY) ? 0.f : mw;
            f[qt][i] = mq_exp2(s_m[wave][row] - m_safe);
        }
    for (int w = 0; w < kMqWaves; ++w) {
        if (wave == w) {
#pragma unroll
            for (int qt = 0; qt < QT; ++qt)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int row = qt * 16 + 4 * kq + i;
#pragma unroll
                    for (int jn = 0; jn < 8; ++jn) {
                        const float v = o[qt][jn][i] * f[qt][i];
                        float *dst = s_acc + row * kMqD + 8 * c + jn;
                        *dst = (w == 0) ? v : *dst + v;
                    }
                }
        }
        __syncthreads();
    }
    // ---- this split's partial
    float *part = p.part + (((bh * p.row_blocks + rb) * (int64_t)p.max_splits + split) * kRows) * kMqPart;
    for (int i = tid; i < kRows * kMqD / 4; i += kMqThreads) {
        const int row = i / (kMqD / 4), q4 = i % (kMqD / 4);
        *reinterpret_cast<float4 *>(part + (int64_t)row * kMqPart + 4 * q4) =
            *reinterpret_cast<const float4 *>(s_acc + row * kMqD + 4 * q4);
    }
    if (tid < kRows) {
        float mw = -INFINITY;
#pragma unroll
        for (int w = 0; w < kMqWaves; ++w) mw = fmaxf(mw, s_m[w][tid]);
        const float m_safe = (mw == -INFINITY) ? 0.f : mw;
        float l = 0.f;
#pragma unroll
        for (int w = 0; w < kMqWaves; ++w) l = fmaf(s_l[w][tid], mq_exp2(s_m[w][tid] - m_safe), l);
        part[(int64_t)tid * kMqPart + kMqD] = mw;
        part[(int64_t)tid * kMqPart + kMqD + 1] = l;
    }
}

// One workgroup of 128 threads per query row of a (sequence, KV head).  The (m, l) of all splits are
// fetched in one trip by the first wavefront (one split per lane) and turned into weights; then every
// thread adds up its output column over the splits, sixteen independent loads at a time.
__global__ __launch_bounds__(kMqD) void multi_attn_combine_kernel(MqParams p) {
    static_assert(kMqMaxSplits <= kWave, "one split per lane of the first wavefront");
    __shared__ float s_w[kMqMaxSplits];
    __shared__ float s_ml[2];
    const int R = blockIdx.x;                 // query row inside the (sequence, KV head): j * G + g
    const int h = blockIdx.y, b = blockIdx.z;
    const int col = threadIdx.x;
    const int64_t bh = (int64_t)b * p.Hkv + h;
    const int rows_total = min(max(p.comp_lens[bh], 0), p.cap) + (p.Kt ? min(max(p.tail_lens[b], 0), p.tail_cap) : 0);
    const int S = mq_splits_for(rows_total, p.max_splits, p.min_rows);
    const int rb = R / p.block_rows, row = R - rb * p.block_rows;
    const float *part = p.part + (((bh * p.row_blocks + rb) * (int64_t)p.max_splits) * p.block_rows + row) * kMqPart;
    const int64_t split_stride = (int64_t)p.block_rows * kMqPart;
    // the first sixteen splits' values of this thread's column are requested together with the (m, l) pairs,
    // not after the weights are known
    float v0[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) v0[k] = (k < S) ? part[k * split_stride + col] : 0.f;
    if (col < kWave) {
        const float m = (col < S) ? part[col * split_stride + kMqD] : -INFINITY;
        const float l = (col < S) ? part[col * split_stride + kMqD + 1] : 0.f;
        float mx = m;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, kWave));
        const float m_safe = (mx == -INFINITY) ? 0.f : mx;
        const float wgt = mq_exp2(m - m_safe);
        float lt = l * wgt;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) lt += __shfl_xor(lt, off, kWave);
        s_w[col] = wgt;
        if (col == 0) { s_ml[0] = mx; s_ml[1] = lt; }
    }
    __syncthreads();
    float acc = 0.f;
#pragma unroll
    for (int k = 0; k < 16; ++k) acc = fmaf(v0[k], (k < S) ? s_w[k] : 0.f, acc);
    for (int s0 = 16; s0 < S; s0 += 16) {
        float v[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) v[k] = (s0 + k < S) ? part[(s0 + k) * split_stride + col] : 0.f;
#pragma unroll
        for (int k = 0; k < 16; ++k) acc = fmaf(v[k], (s0 + k < S) ? s_w[s0 + k] : 0.f, acc);
    }
    const float mx = s_ml[0], l = s_ml[1];
    const int j = R / p.G, g = R - j * p.G;
    const int64_t orow = ((int64_t)j * p.B + b) * p.Hq + (int64_t)h * p.G + g;
    const float out = (l > 0.f) ? acc / l : 0.f;
    if (p.o_is_bf16) reinterpret_cast<uint16_t *>(p.O)[orow * kMqD + col] = (uint16_t)f32_to_bf16(out);
    else reinterpret_cast<float *>(p.O)[orow * kMqD + col] = out;
    if (p.lse && col == 0) p.lse[orow] = (l > 0.f) ? (mx + __log2f(l)) * kMqLn2 : -INFINITY;
}

// ------------------------------------------------------------------------------------------------
static void mq_shape(int B, int Hq, int Hkv, int nq, int cap /* merged + tail rows */, int &row_blocks, int &max_splits, int &min_rows, int &block_rows) {
    const int G = Hq / Hkv;
    // Two tiles of query rows per workgroup read the cache once for 32 rows, but such a workgroup fills a
    // compute unit alone (registers) and a few heads with 17..32 rows do not split into enough of them
    // to cover the chip: those take one tile per workgroup, two row blocks (32 rows, 8 heads, 5 400 cache
    // rows: 14.5 against 17.9 us).
    block_rows = (nq * G <= 16 || (nq * G <= kMqRows && B * Hkv <= 8)) ? 16 : kMqRows;
    if (tuning().multi_block_rows == 16 || tuning().multi_block_rows == 32) block_rows = tuning().multi_block_rows;
    row_blocks = (nq * G + block_rows - 1) / block_rows;
    min_rows = 256;
    // One workgroup per compute unit, never more splits than the capacity can feed: a second round of
    // workgroups waits for the first (measured 15-30 % slower with twice as many), and every split
    // adds a partial per query row that the second kernel reads back.
    const int target = max(1, tuning().multi_target_wgs);
    const int want = (target + B * Hkv * row_blocks - 1) / (B * Hkv * row_blocks);
    const int by_cap = (cap + min_rows - 1) / min_rows;
    max_splits = max(1, min(min(kMqMaxSplits, want), by_cap));
}

static bool mq_fast(const MultiArgs &a) {
    return a.d == kMqD && a.q_dtype == DType::BF16 && a.kv_dtype == DType::BF16;
}

size_t multi_fast_workspace_bytes(int B, int Hq, int Hkv, int nq, int cap) {
    int rb, ms, mr, br;
    mq_shape(B, Hq, Hkv, nq, cap, rb, ms, mr, br);
    return align_up((size_t)B * Hkv * rb * ms * br * kMqPart * 4, 256);
}

size_t multi_workspace_bytes(int B, int Hq, int Hkv, int nq, int cap, int d) {
    const size_t fast = multi_fast_workspace_bytes(B, Hq, Hkv, nq, cap);
    const size_t generic = decode_workspace_bytes(B, Hq, Hkv, cap, d);   // (covers any cap)
    return fast > generic ? fast : generic;
}

hipError_t launch_multi(const MultiArgs &a, hipStream_t stream) {
    if (!mq_fast(a)) {
        // row by row through the decode kernels; their workspace starts with flags that must be zero
        hipError_t e = launch_decode_init_workspace(a.ws, decode_workspace_state_bytes(a.B, a.Hkv), stream);
        if (e != hipSuccess) return e;
        const size_t q_es = a.q_dtype == DType::BF16 ? 2 : 4, o_es = a.o_dtype == DType::BF16 ? 2 : 4;
        const size_t per = (size_t)a.B * a.Hq * a.d;
        for (int j = 0; j < a.nq; ++j) {
            DecodeArgs d;
            d.Q = reinterpret_cast<const char *>(a.Q) + j * per * q_es;
            d.q_dtype = a.q_dtype;
            d.Kc = a.Kc; d.Vc = a.Vc; d.kv_dtype = a.kv_dtype; d.cap = a.cap;
            d.counts = a.counts; d.comp_lens = a.comp_lens;
            d.Kt = a.Kt; d.Vt = a.Vt; d.tail_lens = a.tail_lens; d.tail_cap = a.tail_cap;   // (no mask: checked by the caller)
            d.B = a.B; d.Hq = a.Hq; d.Hkv = a.Hkv; d.d = a.d;
            d.scale = a.scale;
            d.O = reinterpret_cast<char *>(a.O) + j * per * o_es;
            d.o_dtype = a.o_dtype;
            d.lse = a.lse ? a.lse + (size_t)j * a.B * a.Hq : nullptr;
            d.ws = a.ws;
            e = launch_decode(d, stream);
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    }
    return launch_multi_fast(a, stream);
}

hipError_t launch_multi_fast(const MultiArgs &a, hipStream_t stream) {
    MqParams p;
    p.Q = reinterpret_cast<const bf16_t *>(a.Q);
    p.Kc = reinterpret_cast<const bf16_t *>(a.Kc);
    p.Vc = reinterpret_cast<const bf16_t *>(a.Vc);
    p.counts = a.counts; p.comp_lens = a.comp_lens;
    p.Kt = reinterpret_cast<const bf16_t *>(a.Kt);
    p.Vt = reinterpret_cast<const bf16_t *>(a.Vt);
    p.tail_lens = a.tail_lens; p.tail_cap = a.Kt ? a.tail_cap : 0; p.causal = a.causal;
    p.nq = a.nq; p.cap = a.cap; p.B = a.B; p.Hq = a.Hq; p.Hkv = a.Hkv; p.G = a.Hq / a.Hkv;
    p.scale_log2 = a.scale * kMqLog2e;
    p.part = reinterpret_cast<float *>(a.ws);
    mq_shape(a.B, a.Hq, a.Hkv, a.nq, a.cap + p.tail_cap, p.row_blocks, p.max_splits, p.min_rows, p.block_rows);
    p.O = a.O; p.o_is_bf16 = a.o_dtype == DType::BF16; p.lse = a.lse;
    const dim3 grid(p.max_splits, p.row_blocks * a.Hkv, a.B);
    if (p.Kt) {
        if (p.block_rows == 16) hipLaunchKernelGGL((multi_attn_kernel<1, true>), grid, dim3(kMqThreads), 0, stream, p);
        else hipLaunchKernelGGL((multi_attn_kernel<2, true>), grid, dim3(kMqThreads), 0, stream, p);
    } else {
        if (p.block_rows == 16) hipLaunchKernelGGL((multi_attn_kernel<1, false>), grid, dim3(kMqThreads), 0, stream, p);
        else hipLaunchKernelGGL((multi_attn_kernel<2, false>), grid, dim3(kMqThreads), 0, stream, p);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(multi_attn_combine_kernel, dim3(a.nq * p.G, a.Hkv, a.B), dim3(kMqD), 0, stream, p);
    return hipGetLastError();
}

}  // namespace sc
