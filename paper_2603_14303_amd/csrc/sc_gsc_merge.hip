// sc_gsc_merge: Greedy Seed-Based Clustering inside every chunk (paper Sec. 2.3, Alg. 1, Eq. 2)
// followed by mean-pool merging of each cluster (Sec. 2.4, Eq. 3), per (sequence, KV head).
//
// Three kernels:
//   1. gsc_assign  one wavefront per chunk.  The chunk's key rows sit in registers, 8 elements per
//                  lane (d/8 neighbouring lanes cover a row, 64 rows per block).  Seeds are taken in
//                  order; for one seed every lane forms partial dot products for its row pieces, a
//                  transposed DPP reduction hands each lane the full dot product of ONE row, the
//                  cosine is compared with tau and a ballot marks the absorbed rows.  Decisions
//                  inside a +-1e-4 band around tau (and anything involving odd norms) are redone in
//                  fp64 by the whole wave.  Writes the cluster index of every token and the number
//                  of clusters of every chunk.
//   2. gsc_scan    per (sequence, head): exclusive scan over chunks of (clusters + closing
//                  delimiter) -> first output row of every chunk, total rows -> comp_lens.
//   3. gsc_merge   one group of d/8 lanes per OUTPUT row: walks the chunk's cluster indices, gathers
//                  the member rows of its cluster (16-byte pieces, coalesced per row), accumulates in
//                  fp32 in member order, divides by the size and writes the core; delimiter rows and
//                  singletons are copied.
#include "sc_device.h"
#include "sc_gsc_params.h"
#include "sc_host.h"

namespace sc {

// ------------------------------------------------------------------------------------------------
// fp64 re-evaluation of one (seed, candidate) pair by the whole wave: Eq. 2 in double precision.
template <typename T, int D>
__device__ bool cosine_exceeds_f64(const T *seed_row, const T *cand_row, float tau, int lane) {
    double dot = 0.0, ss = 0.0, cc = 0.0;
#pragma unroll
    for (int e = lane; e < D; e += kWave) {
        const double s = load1_f64(seed_row + e), c = load1_f64(cand_row + e);
        dot += s * c; ss += s * s; cc += c * c;
    }
    dot = wave_allreduce_sum(dot);
    ss = wave_allreduce_sum(ss);
    cc = wave_allreduce_sum(cc);
    const double sim = dot / (sqrt(ss) * sqrt(cc));
    return sim > (double)tau;   // NaN compares false: a zero-norm key never merges
}

// ------------------------------------------------------------------------------------------------
// Alg. 1 on one chunk by one wavefront.  Returns the number of clusters.
template <typename T, int D>
__device__ int gsc_chunk(const T *__restrict__ Kbh, int64_t stride_n, int start, int l, float tau,
                         int32_t *__restrict__ cid_bh, int32_t *__restrict__ seed_bh, int lane) {
    constexpr int LPR = D / 8;        // lanes per row
    constexpr int RPW = kWave / LPR;  // rows per wave-wide load
    const int g = lane / LPR, c = lane % LPR;
    // lane r of the wave "owns" block row r; the transposed reduction leaves row RPW*c+g in lane (g,c)
    const int owner_of_my_row = (lane % RPW) * LPR + lane / RPW;

    if (l == 1) {
        if (lane == 0) cid_bh[start] = 0;
        return 1;
    }
    int nseeds = 0;
    for (int rb = 0; rb < l; rb += kWave) {
        const int nr = min(kWave, l - rb);
        const int t_eff = (nr + RPW - 1) / RPW;
        float kreg[LPR][8];
        float part[LPR];
#pragma unroll
        for (int t = 0; t < LPR; ++t) {
            const int row = rb + RPW * t + g;
            if (t < t_eff && row < l) {
                load8(Kbh + (int64_t)(start + row) * stride_n + 8 * c, kreg[t]);
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) kreg[t][e] = 0.f;
            }
            float s = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) s = fmaf(kreg[t][e], kreg[t][e], s);
            part[t] = s;
        }
        const float nsq = lane_gather(row_transpose_reduce<LPR>(part, c), owner_of_my_row);
        const float rinv = __frsqrt_rn(nsq);
        const bool odd_norm = !(nsq > 1e-30f && nsq < 1e30f);

        uint64_t todo = (nr == kWave) ? ~0ull : ((1ull << nr) - 1ull);   // unassigned rows of this block
        int my_cid = -1;
        const int seeds_before = nseeds;
        int old = 0;
        while (todo != 0ull) {
            // next seed: first the seeds of earlier blocks (in order), then the first unassigned row
            int srow, cluster;
            float s_nsq;
            float sreg[8];
            if (old < seeds_before) {
                cluster = old;
                srow = __hip_atomic_load(seed_bh + start + old, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                old += 1;
                load8(Kbh + (int64_t)(start + srow) * stride_n + 8 * c, sreg);
                float s = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) s = fmaf(sreg[e], sreg[e], s);
                s_nsq = row_allreduce_sum<LPR>(s);
            } else {
                const int r = first_bit(todo);
                srow = rb + r;
                cluster = nseeds;
                nseeds += 1;
                if (l > kWave && lane == 0)
                    __hip_atomic_store(seed_bh + start + cluster, srow, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (lane == r) my_cid = cluster;
                todo &= ~(1ull << r);
                s_nsq = __shfl(nsq, r, kWave);
                if (todo == 0ull) break;
                load8(Kbh + (int64_t)(start + srow) * stride_n + 8 * c, sreg);
            }
            const float s_rinv = __frsqrt_rn(s_nsq);
            const bool s_odd = !(s_nsq > 1e-30f && s_nsq < 1e30f);
#pragma unroll
            for (int t = 0; t < LPR; ++t) {
                float s = 0.f;
                if (t < t_eff) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) s = fmaf(kreg[t][e], sreg[e], s);
                }
                part[t] = s;
            }
            const float dotv = lane_gather(row_transpose_reduce<LPR>(part, c), owner_of_my_row);
            const float sim = dotv * rinv * s_rinv;
            const bool cand = (todo >> lane) & 1ull;
            const bool sure_yes = sim > tau + kBand;
            const bool sure_no = sim < tau - kBand;
            const bool unsure = s_odd || odd_norm || !(sure_yes || sure_no);
            bool yes = cand && !unsure && sure_yes;
            uint64_t recheck = ballot64(cand && unsure);
            while (recheck != 0ull) {
                const int j = first_bit(recheck);
                recheck &= recheck - 1ull;
                const bool res = cosine_exceeds_f64<T, D>(Kbh + (int64_t)(start + srow) * stride_n,
                                                          Kbh + (int64_t)(start + rb + j) * stride_n, tau, lane);
                if (lane == j) yes = res;
            }
            const uint64_t absorbed = ballot64(yes);
            if (yes) my_cid = cluster;
            todo &= ~absorbed;
        }
        if (lane < nr) cid_bh[start + rb + lane] = my_cid;
        if (rb + kWave < l) {
            // the seed positions written above are read back by all lanes for the next block
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "agent");
        }
    }
    return nseeds;
}

template <typename T, int D>
__global__ __launch_bounds__(kGscThreads) void gsc_assign_kernel(GscParams p) {
    __shared__ int s_off[kMaxChunksPerItem + 1];
    const int b = blockIdx.z, h = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    // wave index as a scalar: everything derived from it (chunk bounds, loop trip counts) stays
    // wave-uniform for the compiler, so the cross-lane operations below always see all 64 lanes
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int M = p.num_chunks[b];
    if (M <= 0) return;
    int n = p.seq_lens ? p.seq_lens[b] : p.N_max;
    n = n < 0 ? 0 : (n > p.N_max ? p.N_max : n);
    const int C = p.chunks_per_item;
    const int items = (M + C - 1) / C;
    const float tau = p.tau_dev ? *p.tau_dev : p.tau;
    const int64_t bh = (int64_t)b * p.Hkv + h;
    const T *Kbh = reinterpret_cast<const T *>(p.K) + b * p.stride_b + h * p.stride_h;
    const int32_t *off = p.offsets + (int64_t)b * p.offsets_stride_b;
    int32_t *cid_bh = p.cid + bh * p.N_max;
    int32_t *seed_bh = p.seedrow + bh * p.N_max;
    int32_t *pcount_bh = p.pcount + bh * ((int64_t)p.N_max + 1);

    for (int item = blockIdx.x; item < items; item += gridDim.x) {
        const int m0 = item * C;
        const int nch = min(C, M - m0);
        __syncthreads();
        if (tid <= nch) s_off[tid] = off[m0 + tid];
        __syncthreads();
        for (int idx = wave; idx < nch; idx += kGscThreads / kWave) {
            const int start = __builtin_amdgcn_readfirstlane(s_off[idx]);
            const int l = __builtin_amdgcn_readfirstlane(s_off[idx + 1]) - 1 - start;
            int pc = 0;
            if (l > 0) pc = gsc_chunk<T, D>(Kbh, p.stride_n, start, l, tau, cid_bh, seed_bh, lane);
            if (lane == 0) {
                pcount_bh[m0 + idx] = pc;
                const int delim = start + l;
                if (delim < n) cid_bh[delim] = -1;
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// rowbase[m] = rows already present + sum_{m' < m} (pcount[m'] + [chunk m' is closed by a delimiter]);
// comp_lens = total.
__global__ __launch_bounds__(256) void gsc_scan_kernel(GscParams p) {
    __shared__ int s_wave[4];
    __shared__ int s_total;
    const int b = blockIdx.y, h = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int64_t bh = (int64_t)b * p.Hkv + h;
    const int M = p.num_chunks[b];
    if (M <= 0) {
        if (tid == 0) {
            p.comp_lens[bh] = -1;
            if (p.budget) budget_probe_arrive(p.budget, -1, (unsigned int)(p.B * p.Hkv));
        }
        return;
    }
    const int32_t *pcount_bh = p.pcount + bh * ((int64_t)p.N_max + 1);
    int32_t *rowbase_bh = p.rowbase + bh * ((int64_t)p.N_max + 2);
    constexpr int kItems = 8;
    bool base_bad;
    int running = gsc_base_rows(p, bh, base_bad);
    for (int base = 0; base < M; base += 256 * kItems) {
        int v[kItems];
        int sum = 0;
#pragma unroll
        for (int k = 0; k < kItems; ++k) {
            const int m = base + tid * kItems + k;
            v[k] = (m < M) ? (pcount_bh[m] & kPcountMask) + ((m < M - 1) ? 1 : 0) : 0;
            sum += v[k];
        }
        int incl = sum;
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            const int up = __shfl_up(incl, d, kWave);
            if (lane >= d) incl += up;
        }
        if (lane == kWave - 1) s_wave[wave] = incl;
        __syncthreads();
        if (tid == 0) {
            int acc = 0;
            for (int w = 0; w < 4; ++w) { const int t = s_wave[w]; s_wave[w] = acc; acc += t; }
            s_total = acc;
        }
        __syncthreads();
        int excl = running + s_wave[wave] + incl - sum;
#pragma unroll
        for (int k = 0; k < kItems; ++k) {
            const int m = base + tid * kItems + k;
            if (m < M) rowbase_bh[m] = excl;
            excl += v[k];
        }
        running += s_total;
        __syncthreads();
    }
    if (tid == 0) {
        rowbase_bh[M] = running;
        const int rows = (!base_bad && running <= p.cap) ? running : -1;
        p.comp_lens[bh] = rows;
        if (p.budget) budget_probe_arrive(p.budget, rows, (unsigned int)(p.B * p.Hkv));
    }
}

// ------------------------------------------------------------------------------------------------
template <typename TO>
__device__ __forceinline__ void store_row8(void *base, int64_t elem_off, const float (&x)[8]) {
    store8(reinterpret_cast<TO *>(base) + elem_off, x);
}

template <typename T, int D>
__global__ __launch_bounds__(kGscThreads) void gsc_merge_kernel(GscParams p) {
    constexpr int LPR = D / 8;
    constexpr int RPW = kWave / LPR;            // output rows a wave works on at once
    constexpr int kGroups = kGscThreads / LPR;  // output rows a workgroup works on at once
    __shared__ int s_off[kMaxChunksPerItem + 1];
    __shared__ int s_base[kMaxChunksPerItem + 1];
    const int b = blockIdx.z, h = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int g = lane / LPR, c = lane % LPR;
    const int gsh = g * LPR;   // position of this group's bits inside a wave ballot
    const uint64_t gmask = (LPR == 16) ? 0xffffull : 0xffull;
    const int M = p.num_chunks[b];
    if (M <= 0) return;
    int n = p.seq_lens ? p.seq_lens[b] : p.N_max;
    n = n < 0 ? 0 : (n > p.N_max ? p.N_max : n);
    const int C = p.chunks_per_item;
    const int items = (M + C - 1) / C;
    const int64_t bh = (int64_t)b * p.Hkv + h;
    const T *Kbh = reinterpret_cast<const T *>(p.K) + b * p.stride_b + h * p.stride_h;
    const T *Vbh = reinterpret_cast<const T *>(p.V) + b * p.stride_b + h * p.stride_h;
    const int32_t *off = p.offsets + (int64_t)b * p.offsets_stride_b;
    const int32_t *cid_bh = p.cid + bh * p.N_max;
    const int32_t *rowbase_bh = p.rowbase + bh * ((int64_t)p.N_max + 2);
    int32_t *counts_bh = p.counts + bh * p.cap;

    for (int item = blockIdx.x; item < items; item += gridDim.x) {
        const int m0 = item * C;
        const int nch = min(C, M - m0);
        __syncthreads();
        if (tid <= nch) {
            s_off[tid] = off[m0 + tid];
            s_base[tid] = rowbase_bh[m0 + tid];
        }
        __syncthreads();
        const int R0 = __builtin_amdgcn_readfirstlane(s_base[0]);
        const int R1 = min(__builtin_amdgcn_readfirstlane(s_base[nch]), p.cap);
        // all loops below have wave-uniform trip counts; per-group differences are predicates
        for (int Rw = R0 + wave * RPW; Rw < R1; Rw += kGroups) {
            const int R = Rw + g;
            const bool valid = R < R1;
            // chunk of this output row: last idx with s_base[idx] <= R
            int idx = 0;
            for (int k = 1; k < nch; ++k) idx = (s_base[k] <= R) ? k : idx;
            const int start = s_off[idx];
            const int l = s_off[idx + 1] - 1 - start;
            const int cl = R - s_base[idx];
            const bool closed = (start + l) < n;   // chunk is followed by a delimiter
            const int pc = s_base[idx + 1] - s_base[idx] - (closed ? 1 : 0);
            const bool is_delim = valid && cl >= pc;
            const int lscan = (valid && !is_delim) ? l : 0;
            int lmax = 0;
#pragma unroll
            for (int gg = 0; gg < RPW; ++gg) lmax = max(lmax, __builtin_amdgcn_readlane(lscan, gg * LPR));

            float ka[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}, va[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            int size = 0;
            if (is_delim) {
                // the delimiter that closes the chunk: copied unchanged, size 1
                const int64_t src = (int64_t)(start + l) * p.stride_n + 8 * c;
                load8(Kbh + src, ka);
                load8(Vbh + src, va);
                size = 1;
            }
            for (int j0 = 0; j0 < lmax; j0 += LPR) {
                const int j = j0 + c;
                const bool match = (j < lscan) && (cid_bh[start + j] == cl);
                uint32_t mbits = (uint32_t)((ballot64(match) >> gsh) & gmask);
                while (ballot64(mbits != 0u) != 0ull) {
                    int jj[4];
                    bool ok[4];
                    float kk[4][8], vv[4][8];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        ok[u] = mbits != 0u;
                        jj[u] = ok[u] ? (__ffs(mbits) - 1) : 0;
                        mbits &= mbits - 1u;
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        if (ok[u]) {
                            const int64_t src = (int64_t)(start + j0 + jj[u]) * p.stride_n + 8 * c;
                            load8(Kbh + src, kk[u]);
                            load8(Vbh + src, vv[u]);
                        }
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        if (ok[u]) {
                            if (size == 0) {
#pragma unroll
                                for (int e = 0; e < 8; ++e) { ka[e] = kk[u][e]; va[e] = vv[u][e]; }
                            } else {
#pragma unroll
                                for (int e = 0; e < 8; ++e) { ka[e] += kk[u][e]; va[e] += vv[u][e]; }
                            }
                            size += 1;
                        }
                    }
                }
            }
            if (size > 1) {
                const float fs = (float)size;
#pragma unroll
                for (int e = 0; e < 8; ++e) { ka[e] = ka[e] / fs; va[e] = va[e] / fs; }
            }
            if (valid) {
                const int64_t dst = ((int64_t)bh * p.cap + R) * D + 8 * c;
                if (p.out_is_bf16) {
                    store_row8<bf16_t>(p.Kc, dst, ka);
                    store_row8<bf16_t>(p.Vc, dst, va);
                } else {
                    store_row8<float>(p.Kc, dst, ka);
                    store_row8<float>(p.Vc, dst, va);
                }
                if (c == 0) counts_bh[R] = size;
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
size_t gsc_merge_workspace_bytes(int B, int Hkv, int N_max, int d, int out_elem_bytes) {
    const size_t bh = (size_t)B * Hkv;
    size_t bytes = 0;
    bytes += align_up(bh * (size_t)N_max * 4, 256);          // cid
    bytes += align_up(bh * (size_t)N_max * 4, 256);          // seedrow
    bytes += align_up(bh * ((size_t)N_max + 1) * 4, 256);    // pcount
    bytes += align_up(bh * ((size_t)N_max + 2) * 4, 256);    // rowbase
    bytes += align_up(bh * (size_t)N_max * 4, 256);          // stmp
    bytes += 2 * align_up(bh * (size_t)N_max * (size_t)d * (size_t)out_elem_bytes, 256);   // ktmp, vtmp: provisional rows of the output type
    return bytes;
}

hipError_t launch_gsc_scan(const GscParams &p, hipStream_t stream) {
    hipLaunchKernelGGL(gsc_scan_kernel, dim3(p.Hkv, p.B), dim3(256), 0, stream, p);
    return hipGetLastError();
}

template <typename T, int D>
static hipError_t launch_typed(const GscParams &p, hipStream_t stream) {
    const int max_items = (p.N_max + 1 + p.chunks_per_item - 1) / p.chunks_per_item;
    const int gx = max(1, min(max_items, tuning().gsc_grid_x > 0 ? tuning().gsc_grid_x : 128));
    const dim3 grid(gx, p.Hkv, p.B);
    hipLaunchKernelGGL((gsc_assign_kernel<T, D>), grid, dim3(kGscThreads), 0, stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(gsc_scan_kernel, dim3(p.Hkv, p.B), dim3(256), 0, stream, p);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((gsc_merge_kernel<T, D>), grid, dim3(kGscThreads), 0, stream, p);
    return hipGetLastError();
}

// (the fast path addresses a window of rows with 32-bit byte offsets: 64 rows of stride_n elements)
bool gsc_merge_takes_fast_path(const GscMergeArgs &a) {
    return a.in_dtype == DType::BF16 && a.d == 128 && tuning().gsc_fast_path && a.stride_n <= (int64_t(1) << 22);
}

hipError_t launch_gsc_merge(const GscMergeArgs &a, hipStream_t stream) {
    GscParams p;
    p.K = a.K; p.V = a.V;
    p.stride_b = a.stride_b; p.stride_h = a.stride_h; p.stride_n = a.stride_n;
    p.seq_lens = a.seq_lens; p.offsets = a.offsets; p.offsets_stride_b = a.offsets_stride_b;
    p.num_chunks = a.num_chunks;
    p.B = a.B; p.Hkv = a.Hkv; p.N_max = a.N_max;
    p.tau = a.tau;
    p.tau_dev = a.tau_dev;
    p.Kc = a.Kc; p.Vc = a.Vc;
    p.out_is_bf16 = (a.out_dtype == DType::BF16) ? 1 : 0;
    p.cap = a.cap;
    p.counts = a.counts; p.comp_lens = a.comp_lens;
    p.base_lens = a.base_lens;
    p.count_only = a.count_only ? 1 : 0;
    p.budget = nullptr;
    p.chunks_per_item = max(1, min(kMaxChunksPerItem, tuning().gsc_chunks_per_item));

    const size_t bh = (size_t)a.B * a.Hkv;
    char *w = reinterpret_cast<char *>(a.ws);
    int32_t *ws_cid = reinterpret_cast<int32_t *>(w);
    w += align_up(bh * (size_t)a.N_max * 4, 256);
    p.seedrow = reinterpret_cast<int32_t *>(w);
    w += align_up(bh * (size_t)a.N_max * 4, 256);
    p.pcount = reinterpret_cast<int32_t *>(w);
    w += align_up(bh * ((size_t)a.N_max + 1) * 4, 256);
    p.rowbase = reinterpret_cast<int32_t *>(w);
    w += align_up(bh * ((size_t)a.N_max + 2) * 4, 256);
    p.stmp = reinterpret_cast<int32_t *>(w);
    w += align_up(bh * (size_t)a.N_max * 4, 256);
    p.ktmp = w;
    w += align_up(bh * (size_t)a.N_max * (size_t)a.d * (a.out_dtype == DType::BF16 ? 2 : 4), 256);
    p.vtmp = w;
    p.cid = a.cluster_id ? a.cluster_id : ws_cid;
    p.cluster_id = a.cluster_id;

    if (gsc_merge_takes_fast_path(a)) {
        if (a.count_only) p.budget = reinterpret_cast<BudgetState *>(a.budget_state);
        // Two chunks per task pack fuller windows and halve the workgroups; a call so small that every window
        // finds a free wave slot at once (a stretch of tokens appended during decoding) is faster with one,
        // because no window then waits behind another in its workgroup (256 tokens, 8 heads: 19 against 23 us).
        const int auto_chunks = ((int64_t)a.B * a.Hkv * a.N_max <= 32768) ? 1 : 2;
        const int want = tuning().gsc_chunks_per_task > 0 ? tuning().gsc_chunks_per_task : auto_chunks;
        p.chunks_per_item = max(1, min(kMaxChunksPerItem, want));
        return launch_gsc_fast(p, stream);
    }

    if (a.in_dtype == DType::BF16) {
        return a.d == 128 ? launch_typed<bf16_t, 128>(p, stream) : launch_typed<bf16_t, 64>(p, stream);
    }
    return a.d == 128 ? launch_typed<float, 128>(p, stream) : launch_typed<float, 64>(p, stream);
}

}  // namespace sc
