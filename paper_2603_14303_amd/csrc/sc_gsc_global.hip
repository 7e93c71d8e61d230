// sc_gsc_merge_global: Alg. 1 / Eq. 2 and Eq. 3 (paper Sec. 2.3, 2.4) when the whole sequence of a
// (sequence, KV head) is ONE chunk -- the "no chunking" variant of the paper's chunking ablation
// (Sec. 3.4) -- for bf16 keys/values with head dim 128 and up to 32768 tokens.
//
// Alg. 1 over one chunk of n rows is sequential in its seeds (a row is a seed iff no earlier seed takes
// it; a row joins the EARLIEST seed it resembles) but every similarity it can ask for is known in
// advance, so the work is split into a dense part for the whole chip and a short sequential part:
//   norms    reciprocal norms of all rows.
//   pairs    all pairwise comparisons "Sim(i, j) > tau" for i < j on the matrix cores
//            (v_mfma_f32_16x16x32_bf16, 64 x 64 rows per product block): one 64-bit word per (row j,
//            block of 64 earlier rows), "surely above" and "inside the +-1e-4 band" (decided later in
//            fp64), stored column block by column block so that both this kernel and the next one
//            move whole 512-byte runs.  n^2 * d MACs: 69 GMAC and 2 x 67 MB of bits per head at 32k.
//   resolve  one workgroup per (sequence, head) walks the 64-row blocks in order.  Per block: the rows
//            nobody has taken yet run Alg. 1 among themselves on the block's own 64 x 64 bits (one
//            wavefront), then every later row that is still free looks at its word for this block: the
//            first new seed whose bit is set takes it.  Because the blocks come in order, the first
//            seed that takes a row is the earliest one that resembles it, as in Alg. 1.  The same
//            workgroup numbers the members of every cluster in row order.
//   sum      one 16-lane group per cluster adds up its members' keys and values in row order (fp32),
//            scales by 1/size and writes the output row: Eq. 3.
// Everything else (other element types, head dims, longer sequences) is handed to the ordinary kernels
// of sc_gsc_merge with offsets that describe one chunk per sequence.
#include "sc_device.h"
#include "sc_gsc_params.h"
#include "sc_host.h"

#include <mutex>

namespace sc {

typedef float gl_float4 __attribute__((ext_vector_type(4)));
typedef unsigned int gl_u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int gl_u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 gl_bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kGlD = 128;
constexpr int kGlBlock = 64;                    // rows per block
constexpr int kGlTileRowBytes = 272;            // 256 B of keys + 16 B pad: conflict-free operand reads
constexpr int kGlPairWaves = 4;                 // row blocks per workgroup of the pairs kernel
constexpr int kGlResolveThreads = 1024;
constexpr int kGlSegment = 64;                  // column blocks per work item of the pairs kernel
constexpr int kGlList = 32;                     // candidate list entries kept per row

struct GlobParams {
    const bf16_t *K, *V;
    int64_t stride_b, stride_h, stride_n;
    const int32_t *seq_lens;
    int B, Hkv, N_max;
    float tau;
    void *Kc, *Vc;
    int out_is_bf16;
    int cap;
    int32_t *counts, *comp_lens, *cluster_id;
    // workspace, per (sequence, head)
    int nbp;                      // blocks of the longest possible sequence
    long long tri;                // words of one bit array: 64 * nbp * (nbp + 1) / 2
    float *rinv;                  // [nbp * 64]
    unsigned long long *Y, *U;    // [tri]: column block I holds the words of rows 64 I .. 64 nbp - 1
    unsigned char *uflag;         // [nbp][nbp]: (row block J, column block I) has any unsure bit; U is only written (and read) where it has
    int32_t *lists;               // [nbp * 64][kGlList]: earlier rows (of earlier blocks) a row resembles, ascending; bit 31 = unsure
    int32_t *lcount;              // [nbp * 64]: entries of the list (more than kGlList: the list is incomplete, the words decide)
    int32_t *cid, *rank, *order;  // [nbp * 64]
    int32_t *mbase, *csize;       // [nbp * 64 + 1], [nbp * 64]
    int32_t *nclusters;           // [1]
};

__device__ __forceinline__ long long gl_col_base(int I, int nbp) {   // first word of column block I
    return 64ll * ((long long)I * nbp - (long long)I * (I - 1) / 2);
}
__device__ __forceinline__ uint64_t gl_bits_below(int x) {   // bits [0, x), 0 <= x <= 64
    const uint32_t l = (x >= 32) ? 0xFFFFFFFFu : ((1u << x) - 1u);
    const uint32_t h = (x <= 32) ? 0u : ((x >= 64) ? 0xFFFFFFFFu : ((1u << (x - 32)) - 1u));
    return ((uint64_t)h << 32) | l;
}
__device__ __forceinline__ uint32_t gl_or_rows(uint32_t x) {   // OR over the four 16-lane rows, same lane position
    auto r = __builtin_amdgcn_permlane16_swap(x, x, false, false);
    x = r[0] | r[1];
    r = __builtin_amdgcn_permlane32_swap(x, x, false, false);
    return r[0] | r[1];
}
// Eq. 2 in double precision by a whole wavefront (NaN compares false: a zero row resembles nothing)
__device__ __forceinline__ bool gl_cosine_exceeds_f64(const bf16_t *a_row, const bf16_t *b_row, float tau, int lane) {
    double dot = 0.0, aa = 0.0, bb = 0.0;
#pragma unroll
    for (int k = 0; k < kGlD / kWave; ++k) {
        const int e = lane + k * kWave;
        const double a = load1_f64(a_row + e), b = load1_f64(b_row + e);
        dot += a * b; aa += a * a; bb += b * b;
    }
    dot = wave_allreduce_sum(dot);
    aa = wave_allreduce_sum(aa);
    bb = wave_allreduce_sum(bb);
    return dot / (sqrt(aa) * sqrt(bb)) > (double)tau;
}
__device__ __forceinline__ int wave_max_i32(int x) {      // maximum over the wavefront, every lane gets it
    x = max(x, dpp<kDppQuadXor1>(x));
    x = max(x, dpp<kDppQuadXor2>(x));
    x = max(x, dpp<kDppHalfMirror>(x));
    x = max(x, dpp<kDppMirror>(x));
    auto r = __builtin_amdgcn_permlane16_swap((unsigned)x, (unsigned)x, false, false);
    x = max((int)r[0], (int)r[1]);
    r = __builtin_amdgcn_permlane32_swap((unsigned)x, (unsigned)x, false, false);
    return max((int)r[0], (int)r[1]);
}
__device__ __forceinline__ int gl_seq_len(const GlobParams &p, int b) {
    int n = p.seq_lens ? p.seq_lens[b] : p.N_max;
    return n < 0 ? 0 : (n > p.N_max ? p.N_max : n);
}

// ------------------------------------------------------------------------------------------------
// norms: rinv[j] = 1 / |k_j| in fp32 (not a number for rows that do not exist or have an unusable norm:
// every comparison with such a row then lands in the band and is decided in fp64)
__global__ __launch_bounds__(256) void glob_norms_kernel(GlobParams p) {
    const int bh = blockIdx.y, b = bh / p.Hkv, h = bh - b * p.Hkv;
    const int n = gl_seq_len(p, b);
    const int row = blockIdx.x * 16 + threadIdx.x / 16, c = threadIdx.x % 16;
    if (row >= p.nbp * 64) return;
    float nsq = 0.f;
    if (row < n) {
        float x[8];
        load8(p.K + b * p.stride_b + h * p.stride_h + (int64_t)row * p.stride_n + 8 * c, x);
#pragma unroll
        for (int e = 0; e < 8; ++e) nsq = fmaf(x[e], x[e], nsq);
    }
    nsq = row_allreduce_sum<16>(nsq);
    if (c == 0)
        p.rinv[(int64_t)bh * p.nbp * 64 + row] = (row < n && nsq > 1e-30f && nsq < 1e30f) ? __frsqrt_rn(nsq) : __builtin_nanf("");
}

// ------------------------------------------------------------------------------------------------
// pairs: workgroup (JG, bh) owns the row blocks J = 4 JG + wave and walks the column blocks I = 0 .. max J.
// The rows of block J are the B operand and stay in registers (lane (g, c): row 16 Jt + c, elements
// 32 ks + 8 g .. + 7 -- v_mfma_f32_16x16x32_bf16, the form that runs at the full bf16 rate of this chip); the rows of block I pass through an LDS tile shared by the four wavefronts and are
// the A operand.  The product tile leaves lane (g, c) with the dot products of row 16 Jt + c of block J
// and rows 16 It + 4 g + i of block I: four bits of that row's word, completed by an OR over the lane groups.
__global__ __launch_bounds__(kGlPairWaves *kWave, 2) void glob_pairs_kernel(GlobParams p) {
    __shared__ __attribute__((aligned(16))) char s_tiles[2][kGlBlock * kGlTileRowBytes];      // two tiles: one worked on, one being filled
    __shared__ float s_rinvs[2][kGlBlock];
    const int bh = blockIdx.y, b = bh / p.Hkv, h = bh - b * p.Hkv;
    const int n = gl_seq_len(p, b);
    const int nb = (n + kGlBlock - 1) / kGlBlock;
    const int njg = (nb + kGlPairWaves - 1) / kGlPairWaves;
    // Work item = (group JG of four row blocks, segment of kGlSegment column blocks): the walks over the column
    // blocks have about the same length whatever the row.  Groups 16 q .. 16 q + 15 have q + 1 segments each
    // (kGlSegment = 64 column blocks = 16 groups), so 8 q (q + 1) items come before group 16 q.
    int JG, seg;
    {
        const int x = (int)gridDim.x - 1 - (int)blockIdx.x;      // the longest rows first
        int q = 0;
        while (8 * (q + 1) * (q + 2) <= x) ++q;
        const int rem = x - 8 * q * (q + 1);
        JG = 16 * q + rem / (q + 1);
        seg = rem % (q + 1);
    }
    if (JG >= njg) return;
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int g = lane >> 4, c = lane & 15;
    const int J = JG * kGlPairWaves + wave;
    const bool active = J < nb;
    const bf16_t *Kbh = p.K + b * p.stride_b + h * p.stride_h;
    const float *rinv_bh = p.rinv + (int64_t)bh * p.nbp * 64;
    const int sb = (int)p.stride_n * 2;      // bytes between rows
    // rows of block J as B operands, through a descriptor that ends after the sequence's last row
    uint4 bq[4][4];
    float hn[4], wn[4];
    bool bad_j = false;      // a row of block J without a usable norm (also: beyond the end of the sequence)
    {
        const int rows_j = active ? min(kGlBlock, n - J * kGlBlock) : 0;
        const auto src = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(Kbh + (int64_t)(active ? J : 0) * kGlBlock * p.stride_n),
                                                           (short)0, rows_j > 0 ? (rows_j - 1) * sb + kGlD * 2 : 0, 0x00020000);
#pragma unroll
        for (int Jt = 0; Jt < 4; ++Jt) {
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const gl_u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(src, (16 * Jt + c) * sb + (32 * ks + 8 * g) * 2, 0, 0);
                bq[Jt][ks] = make_uint4(v.x, v.y, v.z, v.w);
            }
            const float rn = active ? rinv_bh[J * kGlBlock + 16 * Jt + c] : __builtin_nanf("");
            bad_j = bad_j || !(rn == rn);
            const float norm = __builtin_amdgcn_rcpf(rn);
            hn[Jt] = (p.tau + kBand) * norm;
            wn[Jt] = (2.0f * kBand) * norm;
        }
    }
    bad_j = ballot64(bad_j) != 0ull;
    const int I_first = seg * kGlSegment;
    const int I_last = min(min(JG * kGlPairWaves + kGlPairWaves - 1, nb - 1), I_first + kGlSegment - 1);
    if (I_first > I_last) return;
    // the tile of block I: thread t brings rows t / 16 + 16 r, piece t % 16
    const int lrow = tid >> 4, lc = tid & 15;
    uint4 pre[4];
    float pre_r = 0.f;
    auto fetch = [&](int I) {
        const int rows_i = min(kGlBlock, n - I * kGlBlock);
        const auto src = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(Kbh + (int64_t)I * kGlBlock * p.stride_n), (short)0,
                                                           rows_i > 0 ? (rows_i - 1) * sb + kGlD * 2 : 0, 0x00020000);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const gl_u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(src, (lrow + 16 * r) * sb + 16 * lc, 0, 0);
            pre[r] = make_uint4(v.x, v.y, v.z, v.w);
        }
        if (tid < kGlBlock) pre_r = rinv_bh[I * kGlBlock + tid];
    };
    auto park = [&](int I) {
        char *t = s_tiles[I & 1];
#pragma unroll
        for (int r = 0; r < 4; ++r) *reinterpret_cast<uint4 *>(t + (lrow + 16 * r) * kGlTileRowBytes + 16 * lc) = pre[r];
        if (tid < kGlBlock) s_rinvs[I & 1][tid] = pre_r;
    };
    fetch(I_first);
    park(I_first);
    if (I_first < I_last) fetch(I_first + 1);
    for (int I = I_first; I <= I_last; ++I) {
        __syncthreads();          // tile I is complete; everybody is done with tile I - 1, whose buffer takes tile I + 1 now
        if (I < I_last) {
            park(I + 1);
            if (I + 1 < I_last) fetch(I + 2);      // on its way while this tile is worked on
        }
        const char *s_tile = s_tiles[I & 1];
        const float *s_rinv = s_rinvs[I & 1];
        if (!active || I > J) continue;    // wave-uniform
        uint32_t yl[4], yh[4], ul[4], uh[4];
#pragma unroll
        for (int Jt = 0; Jt < 4; ++Jt) yl[Jt] = yh[Jt] = ul[Jt] = uh[Jt] = 0u;
#pragma unroll
        for (int It = 0; It < 4; ++It) {
            gl_float4 acc[4];
#pragma unroll
            for (int Jt = 0; Jt < 4; ++Jt) acc[Jt] = gl_float4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const uint4 a = *reinterpret_cast<const uint4 *>(s_tile + (16 * It + c) * kGlTileRowBytes + (32 * ks + 8 * g) * 2);
#pragma unroll
                for (int Jt = 0; Jt < 4; ++Jt)
                    acc[Jt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(gl_bf16x8, a),
                                                                      __builtin_bit_cast(gl_bf16x8, bq[Jt][ks]), acc[Jt], 0, 0, 0);
            }
            const gl_float4 rm = *reinterpret_cast<const gl_float4 *>(s_rinv + 16 * It + 4 * g);
            // sim(m, n) > t  <=>  dot * rinv_m > t * norm_n:  dd = (tau + band) * norm_n - dot * rinv_m is negative
            // for a sure yes and at most 2 * band * norm_n inside the band.  Common case, three instructions per
            // pair: the sign bit of dd is shifted into a nibble, an unsigned minimum over the bit patterns keeps the
            // smallest non-negative dd (negative values compare as huge).  Only if some lane saw a value inside
            // the band, or a row without a usable norm is involved, are the nibbles redone with real comparisons
            // (anything that is not a number is "inside the band" and never a sure yes).
            const int sh = 16 * (It & 1) + 4 * g;
            uint32_t yn[4];
            bool close = bad_j || !(rm[0] == rm[0]) || !(rm[1] == rm[1]) || !(rm[2] == rm[2]) || !(rm[3] == rm[3]);
#pragma unroll
            for (int Jt = 0; Jt < 4; ++Jt) {
                uint32_t nib = 0u, dmin = 0x7F800000u;
#pragma unroll
                for (int i = 3; i >= 0; --i) {
                    const uint32_t dd = __float_as_uint(fmaf(-acc[Jt][i], rm[i], hn[Jt]));
                    nib = __builtin_amdgcn_alignbit(nib, dd, 31);      // (nib << 1) | sign bit
                    dmin = min(dmin, dd);
                }
                yn[Jt] = nib;
                close = close || dmin <= __float_as_uint(wn[Jt]);
            }
            if (ballot64(close) != 0ull) {
#pragma unroll
                for (int Jt = 0; Jt < 4; ++Jt) {
                    uint32_t y4 = 0u, u4 = 0u;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float dd = fmaf(-acc[Jt][i], rm[i], hn[Jt]);
                        const bool yes = dd < 0.f;
                        const bool unsure = !yes && !(dd > wn[Jt]);
                        y4 |= yes ? (1u << i) : 0u;
                        u4 |= unsure ? (1u << i) : 0u;
                    }
                    yn[Jt] = y4;
                    if (It < 2) ul[Jt] |= u4 << sh; else uh[Jt] |= u4 << sh;
                }
            }
#pragma unroll
            for (int Jt = 0; Jt < 4; ++Jt) {
                if (It < 2) yl[Jt] |= yn[Jt] << sh; else yh[Jt] |= yn[Jt] << sh;
            }
        }
        // complete the words over the four lane groups; lane 16 Jt + c keeps the words of row 16 Jt + c
        uint32_t myl = 0u, myh = 0u, mul = 0u, muh = 0u;
#pragma unroll
        for (int Jt = 0; Jt < 4; ++Jt) {
            const uint32_t a0 = gl_or_rows(yl[Jt]), a1 = gl_or_rows(yh[Jt]);
            const uint32_t b0 = gl_or_rows(ul[Jt]), b1 = gl_or_rows(uh[Jt]);
            if (g == Jt) { myl = a0; myh = a1; mul = b0; muh = b1; }
        }
        const long long w = (long long)bh * p.tri + gl_col_base(I, p.nbp) + (long long)(J - I) * kGlBlock + lane;
        p.Y[w] = ((unsigned long long)myh << 32) | myl;
        const bool any_u = ballot64((mul | muh) != 0u) != 0ull;
        if (any_u || I == J) p.U[w] = ((unsigned long long)muh << 32) | mul;      // a block's own words are always read
        if (lane == 0) p.uflag[((long long)bh * p.nbp + J) * p.nbp + I] = any_u ? 1 : 0;
    }
}

// ------------------------------------------------------------------------------------------------
// lists: one wavefront per row block J, lane r = row r.  The row's candidates in earlier blocks (set bits
// of its words, column block after column block) in ascending order; bit 31 of an entry = unsure.  The
// first kGlList are kept, the count says how many there were.
__global__ __launch_bounds__(kWave) void glob_lists_kernel(GlobParams p) {
    const int bh = blockIdx.y, b = bh / p.Hkv;
    const int n = gl_seq_len(p, b);
    const int nb = (n + kGlBlock - 1) / kGlBlock;
    const int J = (int)gridDim.x - 1 - (int)blockIdx.x;       // the longest rows first
    if (J >= nb) return;
    const int lane = threadIdx.x, row = J * kGlBlock + lane;
    const unsigned long long *Y = p.Y + (long long)bh * p.tri, *U = p.U + (long long)bh * p.tri;
    const unsigned char *fl = p.uflag + ((long long)bh * p.nbp + J) * p.nbp;
    int32_t *my_list = p.lists + ((int64_t)bh * p.nbp * kGlBlock + row) * kGlList;
    int n_cand = 0;
    constexpr int kBatch = 8;
    for (int I0 = 0; I0 < J; I0 += kBatch) {
        unsigned long long yw[kBatch], uw[kBatch];
#pragma unroll
        for (int k = 0; k < kBatch; ++k) {
            const int I = I0 + k;
            const bool in = I < J;
            const long long w = gl_col_base(in ? I : 0, p.nbp) + (long long)(row - (in ? I : 0) * kGlBlock);
            yw[k] = in ? Y[w] : 0ull;
            uw[k] = (in && fl[in ? I : 0] != 0) ? U[w] : 0ull;
        }
#pragma unroll
        for (int k = 0; k < kBatch; ++k) {
            uint64_t cw = row < n ? (yw[k] | uw[k]) : 0ull;      // rows beyond the end have no list
            while (cw != 0ull) {
                const int bit = first_bit(cw);
                cw &= cw - 1ull;
                if (n_cand < kGlList) my_list[n_cand] = ((I0 + k) * kGlBlock + bit) | (((yw[k] >> bit) & 1ull) ? 0 : (int)0x80000000);
                n_cand += 1;
            }
        }
    }
    if (row < n) p.lcount[(int64_t)bh * p.nbp * kGlBlock + row] = n_cand;
}

// ------------------------------------------------------------------------------------------------
// resolve: one workgroup per (sequence, head) walks the blocks in order; one barrier per block.
//   wavefront 0 (lane r = row r of block J) is the sequential part.  A row that an earlier block's seed
//   resembles is taken by the earliest such seed: the row walks its candidate list (written by the pairs
//   kernel in ascending order) and stops at the first entry that is a seed.  The rows left over run Alg. 1
//   among themselves on the block's own bits; the new seeds go into the seed mask.
//   wavefront 1 brings the lists of block J + 1 into LDS meanwhile (they do not depend on the seeds),
//   wavefront 2 numbers the members of block J - 1 per cluster in row order.
// Unsure candidates (inside the band) are settled by wavefront 0 in fp64, in list order; a row with more
// candidates than the list holds falls back to its words of the bit arrays, column block by column block.
__global__ __launch_bounds__(kGlResolveThreads) void glob_resolve_kernel(GlobParams p) {
    extern __shared__ unsigned short s_csz[];       // members filed per cluster (16 bits: n <= 32768); later their first slot
    __shared__ unsigned long long s_mask[512];      // seeds of every block
    __shared__ int s_pref[513];                     // clusters before block J
    __shared__ int s_list[2][kGlBlock][kGlList + 1];      // [block parity][row][entries]: + 1 keeps the rows on different banks
    __shared__ int s_lcnt[2][kGlBlock];
    __shared__ int s_mine[2][kGlBlock];             // cluster of every row of the block, handed to wavefront 2
    __shared__ int s_scan[kGlResolveThreads];
    const int bh = blockIdx.x, b = bh / p.Hkv, h = bh - b * p.Hkv;
    const int n = gl_seq_len(p, b);
    const int nb = (n + kGlBlock - 1) / kGlBlock;
    const int npad = p.nbp * kGlBlock;
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const bf16_t *Kbh = p.K + b * p.stride_b + h * p.stride_h;
    const unsigned long long *Y = p.Y + (long long)bh * p.tri, *U = p.U + (long long)bh * p.tri;
    const unsigned char *uflag = p.uflag + (long long)bh * p.nbp * p.nbp;
    const int32_t *lists = p.lists + (int64_t)bh * npad * kGlList, *lcount = p.lcount + (int64_t)bh * npad;
    int32_t *cid_g = p.cid + (int64_t)bh * npad, *rank_g = p.rank + (int64_t)bh * npad, *order_g = p.order + (int64_t)bh * npad;
    int32_t *cid_out = p.cluster_id ? p.cluster_id + (int64_t)bh * p.N_max : nullptr;
    for (int i = tid; i < npad; i += kGlResolveThreads) s_csz[i] = 0;
    if (tid == 0) s_pref[0] = 0;
    if (tid < kGlBlock) s_lcnt[0][tid] = 0;      // block 0 has no earlier block
    __syncthreads();

    // wavefront 0: words of block J's rows in its own column block
    unsigned long long dy = 0ull, du = 0ull;
    if (wave == 0 && nb > 0) { dy = Y[lane]; du = U[lane]; }
    for (int J = 0; J <= nb; ++J) {      // one extra step: wavefront 2 files the last block
        if (wave == 0 && J < nb) {
            const int j = J * kGlBlock + lane;
            const bool valid = j < n;
            // ---- earliest seed of an earlier block that resembles the row
            const int cnt = valid ? s_lcnt[J & 1][lane] : 0;
            int seed_row = -1;
            bool slow = false;
            {
                // the list holds the row's kGlList earliest candidates: if one of them is a seed, the earliest seed
                // is among them; if none is and the list is incomplete, the words decide
                const int cmax = __builtin_amdgcn_readfirstlane(wave_max_i32(min(cnt, kGlList)));
                bool done = false;
                for (int e = 0; e < cmax; ++e) {
                    const int ent = s_list[J & 1][lane][e];
                    const int i = (e < cnt) ? (ent & 0x7FFFFFFF) : 0;      // beyond the list: whatever the buffer held before
                    const bool is_seed = !done && e < cnt && ((s_mask[i >> 6] >> (i & 63)) & 1ull) != 0ull;
                    if (is_seed) {
                        done = true;
                        if (ent >= 0) seed_row = i;      // sure
                        else slow = true;                // unsure: decided below, in list order
                    }
                }
                if (!done && cnt > kGlList) slow = true;
            }
            uint64_t slow_rows = ballot64(slow);
            while (slow_rows != 0ull) {
                const int r = __builtin_amdgcn_readfirstlane(first_bit(slow_rows));
                slow_rows &= slow_rows - 1ull;
                const int jr = J * kGlBlock + r;
                const int cr = __builtin_amdgcn_readlane(cnt, r);
                int found = -1;
                for (int e = 0; e < min(cr, kGlList) && found < 0; ++e) {
                    const int ent = s_list[J & 1][r][e];
                    const int i = ent & 0x7FFFFFFF;
                    if (((s_mask[i >> 6] >> (i & 63)) & 1ull) == 0ull) continue;
                    bool ok = ent >= 0;
                    if (!ok) ok = gl_cosine_exceeds_f64(Kbh + (int64_t)i * p.stride_n, Kbh + (int64_t)jr * p.stride_n, p.tau, lane);
                    if (ok) found = i;
                }
                if (found < 0 && cr > kGlList) {
                    for (int I0 = 0; I0 < J && found < 0; I0 += kWave) {
                        const int I = I0 + lane;
                        unsigned long long yy = 0ull, cc = 0ull;
                        if (I < J) {
                            const long long w = gl_col_base(I, p.nbp) + (long long)(jr - I * kGlBlock);
                            const unsigned long long m = s_mask[I];
                            yy = Y[w] & m;
                            cc = yy | (uflag[(long long)J * p.nbp + I] ? (U[w] & m) : 0ull);
                        }
                        uint64_t cols = ballot64(cc != 0ull);
                        while (cols != 0ull && found < 0) {
                            const int l = __builtin_amdgcn_readfirstlane(first_bit(cols));
                            cols &= cols - 1ull;
                            const unsigned long long ycol = __builtin_bit_cast(unsigned long long, make_uint2(
                                __builtin_amdgcn_readlane((unsigned)yy, l), __builtin_amdgcn_readlane((unsigned)(yy >> 32), l)));
                            unsigned long long ccol = __builtin_bit_cast(unsigned long long, make_uint2(
                                __builtin_amdgcn_readlane((unsigned)cc, l), __builtin_amdgcn_readlane((unsigned)(cc >> 32), l)));
                            while (ccol != 0ull && found < 0) {
                                const int bit = first_bit(ccol);
                                ccol &= ccol - 1ull;
                                const int srow = (I0 + l) * kGlBlock + bit;
                                bool ok = ((ycol >> bit) & 1ull) != 0ull;
                                if (!ok) ok = gl_cosine_exceeds_f64(Kbh + (int64_t)srow * p.stride_n, Kbh + (int64_t)jr * p.stride_n, p.tau, lane);
                                if (ok) found = srow;
                            }
                        }
                    }
                }
                if (lane == r) seed_row = found;
            }
            int mine = -1;
            if (seed_row >= 0) {
                const int I = seed_row >> 6, bit = seed_row & 63;
                mine = s_pref[I] + __popcll(s_mask[I] & gl_bits_below(bit));
            }
            // ---- Alg. 1 among the rows of block J that nobody has taken
            const bool open = valid && seed_row < 0;
            const uint64_t y = dy & gl_bits_below(lane), u = du & gl_bits_below(lane);
            uint64_t todo = ballot64(open), seeds = 0ull;
            int my_seed = 0;
            {
                // Shortcut: guess that a free row is a seed iff no earlier free row of the block resembles it.  If every
                // other free row then resembles an earlier guessed seed, and no unsure pair is involved, induction over
                // the rows shows that the guess is the outcome of Alg. 1 (a guessed seed has no earlier similar free
                // row, hence no earlier similar seed; any other row joins the first guessed seed it resembles).
                const uint64_t free_before = todo & gl_bits_below(lane);
                const bool guess = open && (y & free_before) == 0ull;
                const uint64_t S = ballot64(guess);
                const uint64_t hits = y & S;
                const bool fine = !open || ((u & free_before) == 0ull && (guess || hits != 0ull));
                if (ballot64(fine) == ~0ull) {
                    seeds = S;
                    my_seed = guess ? lane : (hits != 0ull ? first_bit(hits) : 0);
                    todo = 0ull;
                }
            }
            while (todo != 0ull) {
                const int s = __builtin_amdgcn_readfirstlane(first_bit(todo));     // lowest free row: nobody before it took it
                const bool cand = ((todo >> lane) & 1ull) != 0ull && lane > s;
                bool yes = cand && ((y >> s) & 1ull) != 0ull;
                uint64_t recheck = ballot64(cand && !yes && ((u >> s) & 1ull) != 0ull);
                while (recheck != 0ull) {
                    const int jl = __builtin_amdgcn_readfirstlane(first_bit(recheck));
                    recheck &= recheck - 1ull;
                    const bool res = gl_cosine_exceeds_f64(Kbh + (int64_t)(J * kGlBlock + s) * p.stride_n,
                                                           Kbh + (int64_t)(J * kGlBlock + jl) * p.stride_n, p.tau, lane);
                    if (lane == jl) yes = res;
                }
                const uint64_t got = ballot64(yes);
                if (lane == s || yes) my_seed = s;
                seeds |= 1ull << s;
                todo &= ~(got | (1ull << s));
            }
            const int first = s_pref[J];
            if (open) mine = first + __popcll(seeds & gl_bits_below(my_seed));
            if (lane == 0) { s_mask[J] = seeds; s_pref[J + 1] = first + __popcll(seeds); }
            s_mine[J & 1][lane] = valid ? mine : -1;
            // the next block's own words, requested now, used after the barrier
            if (J + 1 < nb) {
                const long long w = gl_col_base(J + 1, p.nbp) + lane;
                dy = Y[w];
                du = U[w];
            }
        } else if (wave == 1 && J + 1 < nb) {
            // ---- lists of block J + 1 into LDS
            const int T = J + 1, jrow = T * kGlBlock + lane;
            const int cnt = jrow < n ? lcount[jrow] : 0;
            s_lcnt[T & 1][lane] = cnt;
            // 64 rows x 32 entries, 16 bytes per lane and load
#pragma unroll
            for (int q = 0; q < (kGlBlock * kGlList) / (kWave * 4); ++q) {
                const int flat = (q * kWave + lane) * 4;            // entry index inside the block's 64 x 32 array
                const int r = flat / kGlList, e = flat % kGlList;
                const int4 v = *reinterpret_cast<const int4 *>(lists + ((int64_t)T * kGlBlock + r) * kGlList + e);
                s_list[T & 1][r][e] = v.x; s_list[T & 1][r][e + 1] = v.y; s_list[T & 1][r][e + 2] = v.z; s_list[T & 1][r][e + 3] = v.w;
            }
        } else if (wave == 2 && J >= 1) {
            // ---- members of block J - 1 in row order
            const int Jb = J - 1, j = Jb * kGlBlock + lane;
            const bool valid = j < n;
            const int mine = s_mine[Jb & 1][lane];
            if (valid) {
                cid_g[j] = mine;
                if (cid_out) cid_out[j] = mine;
            }
            // rank of row j among the members of its cluster = members filed so far + earlier rows of this block in
            // the same cluster.  All lanes read the old sizes first, then the first row of every cluster in the block
            // files the new size (distinct clusters, distinct addresses): no chain of dependent LDS updates.
            int lower = 0, total = 0;
            uint64_t rem = ballot64(valid);
            while (rem != 0ull) {      // once per cluster that has rows in the block
                const int l0 = __builtin_amdgcn_readfirstlane(first_bit(rem));
                const int c0 = __builtin_amdgcn_readlane(mine, l0);
                const uint64_t same = ballot64(valid && mine == c0);
                if ((same >> lane) & 1ull) { lower = __popcll(same & gl_bits_below(lane)); total = __popcll(same); }
                rem &= ~same;
            }
            const int before = valid ? (int)s_csz[mine] : 0;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
            if (valid && lower == 0) s_csz[mine] = (unsigned short)(before + total);
            if (valid) rank_g[j] = before + lower;
        }
        __syncthreads();
    }
    // ---- cluster sizes -> first member slot of every cluster; sizes and length to the outputs
    const int P = s_pref[nb];
    {
        constexpr int kPer = 32;             // 1024 threads x 32 = 32768 clusters at most
        int local[kPer];
        int sum = 0;
#pragma unroll
        for (int k = 0; k < kPer; ++k) {
            const int cidx = tid * kPer + k;
            local[k] = (cidx < P) ? (int)s_csz[cidx] : 0;
            sum += local[k];
        }
        s_scan[tid] = sum;
        __syncthreads();
        for (int off = 1; off < kGlResolveThreads; off <<= 1) {
            const int v = (tid >= off) ? s_scan[tid - off] : 0;
            __syncthreads();
            s_scan[tid] += v;
            __syncthreads();
        }
        int run = s_scan[tid] - sum;
        int32_t *mbase = p.mbase + (int64_t)bh * (npad + 1), *csize = p.csize + (int64_t)bh * npad;
        int32_t *counts_bh = p.counts + (int64_t)bh * p.cap;
#pragma unroll
        for (int k = 0; k < kPer; ++k) {
            const int cidx = tid * kPer + k;
            if (cidx < P) {
                mbase[cidx] = run;
                csize[cidx] = local[k];
                if (cidx < p.cap) counts_bh[cidx] = local[k];
                s_csz[cidx] = (unsigned short)run;      // n <= 32768: a slot index fits 16 bits
                run += local[k];
            }
        }
        if (tid == 0) {
            p.nclusters[bh] = P;
            p.comp_lens[bh] = (P <= p.cap) ? P : -1;
        }
    }
    __syncthreads();
    for (int j = tid; j < n; j += kGlResolveThreads) order_g[(int)s_csz[cid_g[j]] + rank_g[j]] = j;
}

// ------------------------------------------------------------------------------------------------
// sum: Eq. 3.  16 lanes per cluster, members in row order, four rows in flight.
template <typename TO>
__global__ __launch_bounds__(256) void glob_sum_kernel(GlobParams p) {
    const int bh = blockIdx.y, b = bh / p.Hkv, h = bh - b * p.Hkv;
    const int npad = p.nbp * kGlBlock;
    const int P = min(p.nclusters[bh], p.cap);
    const int cl = blockIdx.x * 16 + threadIdx.x / 16, c = threadIdx.x % 16;
    if (cl >= P) return;
    const bf16_t *Kbh = p.K + b * p.stride_b + h * p.stride_h + 8 * c;
    const bf16_t *Vbh = p.V + b * p.stride_b + h * p.stride_h + 8 * c;
    const int32_t *order = p.order + (int64_t)bh * npad + p.mbase[(int64_t)bh * (npad + 1) + cl];
    const int size = p.csize[(int64_t)bh * npad + cl];
    float ka[8], va[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) ka[e] = va[e] = 0.f;
    for (int t0 = 0; t0 < size; t0 += 4) {
        float kk[4][8], vv[4][8];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (t0 + u < size) {
                const int64_t row = order[t0 + u];
                load8(Kbh + row * p.stride_n, kk[u]);
                load8(Vbh + row * p.stride_n, vv[u]);
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (t0 + u < size) {
#pragma unroll
                for (int e = 0; e < 8; ++e) { ka[e] += kk[u][e]; va[e] += vv[u][e]; }
            }
        }
    }
    // 1/size: a row of size 1 is passed on unchanged
    const float inv = (size > 1) ? 1.0f / (float)size : 1.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) { ka[e] *= inv; va[e] *= inv; }
    TO *Kc = reinterpret_cast<TO *>(p.Kc) + ((int64_t)bh * p.cap + cl) * kGlD + 8 * c;
    TO *Vc = reinterpret_cast<TO *>(p.Vc) + ((int64_t)bh * p.cap + cl) * kGlD + 8 * c;
    store8(Kc, ka);
    store8(Vc, va);
}

// one chunk per sequence in the offsets format of sc_segment: off = {0, n + 1}, one chunk
__global__ void glob_one_chunk_kernel(const int32_t *seq_lens, int B, int N_max, int32_t *offsets, int32_t *num_chunks) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    int n = seq_lens ? seq_lens[b] : N_max;
    n = n < 0 ? 0 : (n > N_max ? N_max : n);
    offsets[2 * b] = 0;
    offsets[2 * b + 1] = n + 1;
    num_chunks[b] = 1;
}

// ------------------------------------------------------------------------------------------------
static bool glob_fast_ok(const GscMergeArgs &a) {
    return a.in_dtype == DType::BF16 && a.d == kGlD && a.N_max <= 32768 && a.stride_n % 8 == 0 && a.stride_n * 2 * kGlBlock < (1ll << 31) &&
           tuning().gsc_fast_path != 0;
}
static size_t glob_head_bytes(int N_max) {   // upper bound of what launch_gsc_global lays out per (sequence, head)
    const size_t nbp = (size_t)(N_max + kGlBlock - 1) / kGlBlock, npad = nbp * kGlBlock;
    const size_t tri = 64 * nbp * (nbp + 1) / 2;
    return 6 * align_up(npad * 4, 256) + 2 * align_up(tri * 8, 256) + align_up((npad + 1) * 4, 256) + align_up(nbp * nbp, 256) +
           align_up(npad * kGlList * 4, 256);
}
// workspace: [one-chunk offsets and counts | the larger of (ordinary sc_gsc_merge workspace, arrays of this path)]
static size_t glob_prefix_bytes(int B) { return align_up((size_t)B * 3 * 4, 256); }

size_t gsc_global_workspace_bytes(int B, int Hkv, int N_max, int d) {
    const size_t ordinary = gsc_merge_workspace_bytes(B, Hkv, N_max, d);
    size_t fast = 0;
    if (d == kGlD && N_max <= 32768) {
        fast = glob_head_bytes(N_max) * (size_t)B * Hkv + align_up((size_t)B * Hkv * 4, 256);
    }
    return glob_prefix_bytes(B) + (ordinary > fast ? ordinary : fast);
}

hipError_t launch_gsc_global(const GscMergeArgs &a, hipStream_t stream) {
    char *ws = reinterpret_cast<char *>(a.ws);
    int32_t *offsets = reinterpret_cast<int32_t *>(ws), *num_chunks = offsets + 2 * a.B;
    char *rest = ws + glob_prefix_bytes(a.B);
    if (!glob_fast_ok(a)) {
        hipLaunchKernelGGL(glob_one_chunk_kernel, dim3((a.B + 255) / 256), dim3(256), 0, stream, a.seq_lens, a.B, a.N_max, offsets, num_chunks);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        GscMergeArgs o = a;
        o.offsets = offsets; o.offsets_stride_b = 2; o.num_chunks = num_chunks; o.ws = rest;
        return launch_gsc_merge(o, stream);
    }
    GlobParams p;
    p.K = reinterpret_cast<const bf16_t *>(a.K); p.V = reinterpret_cast<const bf16_t *>(a.V);
    p.stride_b = a.stride_b; p.stride_h = a.stride_h; p.stride_n = a.stride_n;
    p.seq_lens = a.seq_lens; p.B = a.B; p.Hkv = a.Hkv; p.N_max = a.N_max; p.tau = a.tau;
    p.Kc = a.Kc; p.Vc = a.Vc; p.out_is_bf16 = a.out_dtype == DType::BF16; p.cap = a.cap;
    p.counts = a.counts; p.comp_lens = a.comp_lens; p.cluster_id = a.cluster_id;
    p.nbp = (a.N_max + kGlBlock - 1) / kGlBlock;
    p.tri = 64ll * p.nbp * (p.nbp + 1) / 2;
    const size_t BH = (size_t)a.B * a.Hkv;
    const size_t npad = (size_t)p.nbp * kGlBlock;
    // array by array, each holding all (sequence, head) pairs back to back
    size_t o = 0;
    p.rinv = reinterpret_cast<float *>(rest + o); o += align_up(npad * 4 * BH, 256);
    p.Y = reinterpret_cast<unsigned long long *>(rest + o); o += align_up((size_t)p.tri * 8 * BH, 256);
    p.U = reinterpret_cast<unsigned long long *>(rest + o); o += align_up((size_t)p.tri * 8 * BH, 256);
    p.cid = reinterpret_cast<int32_t *>(rest + o); o += align_up(npad * 4 * BH, 256);
    p.rank = reinterpret_cast<int32_t *>(rest + o); o += align_up(npad * 4 * BH, 256);
    p.order = reinterpret_cast<int32_t *>(rest + o); o += align_up(npad * 4 * BH, 256);
    p.mbase = reinterpret_cast<int32_t *>(rest + o); o += align_up((npad + 1) * 4 * BH, 256);
    p.csize = reinterpret_cast<int32_t *>(rest + o); o += align_up(npad * 4 * BH, 256);
    p.nclusters = reinterpret_cast<int32_t *>(rest + o); o += align_up(4 * BH, 256);
    p.uflag = reinterpret_cast<unsigned char *>(rest + o); o += align_up((size_t)p.nbp * p.nbp * BH, 256);
    p.lists = reinterpret_cast<int32_t *>(rest + o); o += align_up(npad * kGlList * 4 * BH, 256);
    p.lcount = reinterpret_cast<int32_t *>(rest + o); o += align_up(npad * 4 * BH, 256);

    hipLaunchKernelGGL(glob_norms_kernel, dim3((unsigned)(npad / 16), (unsigned)BH), dim3(256), 0, stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int njg = (p.nbp + kGlPairWaves - 1) / kGlPairWaves;
    int items = 0;      // see the kernel: group JG has JG / 16 + 1 segments
    for (int jg = 0; jg < njg; ++jg) items += jg / 16 + 1;
    hipLaunchKernelGGL(glob_pairs_kernel, dim3((unsigned)items, (unsigned)BH), dim3(kGlPairWaves * kWave), 0, stream, p);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(glob_lists_kernel, dim3((unsigned)p.nbp, (unsigned)BH), dim3(kWave), 0, stream, p);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    const size_t dyn = npad * sizeof(unsigned short);
    if (dyn > 48 * 1024) {   // a host-side setting of the kernel (per device), not a stream operation
        int dev = 0;
        e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        static std::mutex mu;
        static bool raised[64];
        if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
        std::lock_guard<std::mutex> lock(mu);
        if (!raised[dev]) {
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(glob_resolve_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024);
            if (e != hipSuccess) return e;
            raised[dev] = true;
        }
    }
    hipLaunchKernelGGL(glob_resolve_kernel, dim3((unsigned)BH), dim3(kGlResolveThreads), dyn, stream, p);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int max_clusters = a.N_max < a.cap ? a.N_max : a.cap;
    const dim3 grid_sum((unsigned)((max_clusters + 15) / 16), (unsigned)BH);
    if (p.out_is_bf16) hipLaunchKernelGGL((glob_sum_kernel<bf16_t>), grid_sum, dim3(256), 0, stream, p);
    else hipLaunchKernelGGL((glob_sum_kernel<float>), grid_sum, dim3(256), 0, stream, p);
    return hipGetLastError();
}

}  // namespace sc
