// Fast path of sc_gsc_merge for bf16 keys/values with head dim 128 (paper Sec. 2.3 Alg. 1 / Eq. 2 and
// Sec. 2.4 Eq. 3).
//
// Two launches (three for sequences of more than 32k tokens):
//   compress  reads K and V once.  One single-wavefront workgroup handles a task of one or two consecutive
//           chunks.  It packs whole chunks (each with its closing delimiter) into "windows" of at most 64
//           rows.  Keys and values of a window are loaded together (16 lanes per row, 16-byte
//           pieces); the keys are parked in LDS, the values wait in registers.  All pairwise
//           cosines of the window come from one Gram matrix on the matrix cores, are compared with
//           tau (decisions inside +-1e-4 of tau are redone in fp64 where they matter) and filed as a bit
//           matrix, on which the seed set of Alg. 1 is found as the fixed point of the first-fit rule
//           (a few bit operations per application; seed by seed as the fallback).  A delimiter is
//           a one-row chunk, so the seeds in row order ARE the output rows of the window.  The
//           cluster means are a second small matrix product: (output row x window row) 0/1
//           membership times (window row x 128) keys or values, fp32 accumulate, with a ones column
//           giving the sizes.  Results go to provisional rows (the window's own first rows), because
//           the final row of a window depends on every window before it.
//   scan      (beyond 32k tokens only; shorter sequences add the counts up inside relocate) exclusive scan of
//           (clusters + delimiter) over the chunks of a (sequence, head).
//   relocate  moves the merged rows and sizes from their provisional to their final rows.
// A chunk longer than one window runs over several 64-row blocks with its seeds carried along: the first
// sixteen in registers, further ones re-read through L2.
#include "sc_device.h"
#include "sc_gsc_params.h"
#include "sc_host.h"

namespace sc {

typedef __bf16 bf16x8f_t __attribute__((ext_vector_type(8)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));


constexpr int kFastD = 128;
constexpr int kWin = 64;                 // rows of a window
constexpr float kFastBand = 1e-4f;       // fp32 cosine error for d = 128 is < 2e-5; inside the band -> fp64

__device__ __forceinline__ uint64_t bits_range(int lo, int hi) {   // bits [lo, hi), 0 <= lo <= hi <= 64
    const uint64_t upto_hi = (hi >= 64) ? ~0ull : ((1ull << hi) - 1ull);
    const uint64_t upto_lo = (lo >= 64) ? ~0ull : ((1ull << lo) - 1ull);
    return upto_hi & ~upto_lo;
}
__device__ __forceinline__ uint64_t bits_below(int x) {   // bits [0, x), 0 <= x <= 64, from 32-bit operations
    const uint32_t l = (x >= 32) ? 0xFFFFFFFFu : ((1u << x) - 1u);
    const uint32_t h = (x <= 32) ? 0u : ((x >= 64) ? 0xFFFFFFFFu : ((1u << (x - 32)) - 1u));
    return ((uint64_t)h << 32) | l;
}

// LDS layout of a wavefront
constexpr int kLdsRowBytes = 272;                         // 256 B of keys + 16 B pad: conflict-free tile reads
constexpr int kLdsRinvOff = kWin * kLdsRowBytes;          // 64 reciprocal norms
constexpr int kLdsBitsOff = kLdsRinvOff + 256;            // per row: yes lo/hi, unsure lo/hi (16 B)
constexpr int kLdsIdxOff = kLdsBitsOff + kWin * 16;       // 64 output-index bytes
constexpr int kLdsSeedRinvOff = kLdsIdxOff + 64;          // reciprocal norms of the first 16 seeds of a long chunk
constexpr int kLdsWaveBytes = kLdsSeedRinvOff + 64;

__device__ __forceinline__ void wave_lds_fence() {
    // LDS traffic of one wavefront executes in order; this only stops the compiler from moving
    // accesses of other lanes' data across the hand-over point
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

// Rows of a window / block as loaded: lane (g = lane/16, c = lane%16) holds elements 8c..8c+7 of rows
// 4t + g, t = 0..15 (one coalesced 16-byte load per t covers four whole rows).
struct RowRegs {
    uint4 r[16];
};

typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
// cache policy of the key/value row loads: nt = read once by this launch.  Every input row is read exactly once;
// without the hint the rows displace the provisional rows (which the relocation reads back) from the caches
// (32k-token layer: 54.7 -> 50.7 us per call; with it the relocation's own reads and writes carry the hint too)
constexpr int kAuxReadOnce = 2;

// Rows [first_row, first_row + nrows) through a buffer descriptor that ends after the last wanted row:
// the hardware returns zeros for every access beyond it, so no lane needs a predicate or a 64-bit
// address.  row_stride_bytes * 64 must fit in 31 bits (checked by the launcher).
struct RowSource {
    __amdgpu_buffer_rsrc_t rsrc;
    int voff;     // this lane's offset inside a group of four rows: g * stride + 16 * c
    int step;     // four rows further: 4 * stride
};
__device__ __forceinline__ RowSource row_source(const bf16_t *base, int64_t stride_n, int first_row, int nrows, int g, int c) {
    RowSource rs;
    const int sb = (int)stride_n * 2;
    rs.rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(base + (int64_t)first_row * stride_n), (short)0,
                                                nrows > 0 ? (nrows - 1) * sb + kFastD * 2 : 0, 0x00020000);
    rs.voff = g * sb + 16 * c;
    rs.step = 4 * sb;
    return rs;
}
__device__ __forceinline__ void load_rows(RowRegs &x, const RowSource &rs) {
#pragma unroll
    for (int t = 0; t < 16; ++t) {
        const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(rs.rsrc, rs.voff + t * rs.step, 0, kAuxReadOnce);
        x.r[t] = make_uint4(v.x, v.y, v.z, v.w);
    }
}

// fp64 re-evaluation of one (seed, candidate) pair by the whole wave: Eq. 2 in double precision
__device__ __forceinline__ bool cosine_exceeds_f64_fast(const bf16_t *seed_row, const bf16_t *cand_row, float tau, int lane) {
    double dot = 0.0, ss = 0.0, cc = 0.0;
#pragma unroll
    for (int k = 0; k < kFastD / kWave; ++k) {
        const int e = (lane & (kWave - 1)) + k * kWave;
        const double s = load1_f64(seed_row + e), c = load1_f64(cand_row + e);
        dot += s * c; ss += s * s; cc += c * c;
    }
    dot = wave_allreduce_sum(dot);
    ss = wave_allreduce_sum(ss);
    cc = wave_allreduce_sum(cc);
    return dot / (sqrt(ss) * sqrt(cc)) > (double)tau;   // NaN compares false
}

// the same for two rows of the window / block parked in LDS by gram_bitmatrix (the parked bf16 values are
// the inputs themselves, so the result is the same; the rows come back in a tenth of the time of a
// trip to memory, which matters when tau lies inside the band of the similarities and many pairs are redone)
__device__ __forceinline__ bool cosine_exceeds_f64_lds(const char *lds, int row_a, int row_b, float tau, int lane);

__device__ __forceinline__ float safe_rinv(float nsq) {
    // a norm that is zero, denormal, huge or not a number makes every cosine with that row "unsure"
    return (nsq > 1e-30f && nsq < 1e30f) ? __frsqrt_rn(nsq) : __builtin_nanf("");
}

// ------------------------------------------------------------------------------------------------
// Membership products on the matrix cores (Eq. 3 as a 0/1 matrix times the rows): membership_mfma_tiles and
// membership_mfma_kv below.
// scale the sums of tile `ot` by 1/size and store rows [16*ot, 16*ot+16) ∩ [0, n_out) at dst_row0 + o
template <typename TO>
__device__ __forceinline__ void store_tile(const floatx4_t (&D)[8], const floatx4_t &Dn, int ot, int n_out, TO *dst,
                                           int64_t dst_row0, int64_t row_limit, int lane) {
    const int g = lane >> 4;
    // The provisional rows are read by the next launch from any chiplet: they are written through to the
    // memory side (sc1) instead of staying dirty in this chiplet's L2 until the kernel ends.  dst is
    // wave-uniform; its rows from dst_row0 on behind a descriptor, the lane's piece as offset.
    constexpr int kRowBytes = kFastD * (int)sizeof(TO);
    const int rows_left = (int)min(row_limit - dst_row0, (int64_t)(1 << 21));      // (n_out rows at most are stored)
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(dst + dst_row0 * kFastD, (short)0, rows_left * kRowBytes, 0x00020000);
    constexpr int kAuxThrough = 16;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int o = 16 * ot + 4 * g + i;
        if (o < n_out && dst_row0 + o < row_limit) {
            // 1/size: exact for powers of two, 1 ulp otherwise; a row of size 1 is multiplied by exactly 1
            const float inv = (Dn[i] > 1.5f) ? __builtin_amdgcn_rcpf(Dn[i]) : 1.0f;
            float v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = D[j][i] * inv;
            const int off = o * kRowBytes + 8 * (lane & 15) * (int)sizeof(TO);
            if constexpr (sizeof(TO) == 2) {
                const u32x4_t t = {pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7])};
                __builtin_amdgcn_raw_buffer_store_b128(t, rs, off, 0, kAuxThrough);
            } else {
                const u32x4_t t0 = {__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])};
                const u32x4_t t1 = {__float_as_uint(v[4]), __float_as_uint(v[5]), __float_as_uint(v[6]), __float_as_uint(v[7])};
                __builtin_amdgcn_raw_buffer_store_b128(t0, rs, off, 0, kAuxThrough);
                __builtin_amdgcn_raw_buffer_store_b128(t1, rs, off + 16, 0, kAuxThrough);
            }
        }
    }
}



// output indices as bytes (0xFF = none) in the operand order of the membership product:
// ob[q] byte i = index of row 16q + 4i + lane/16
__device__ __forceinline__ void orow_to_operand_bytes(int rel_o, int lane, uint32_t (&ob)[4]) {
    const int g = lane >> 4;
    const int v = (rel_o >= 0 && rel_o < 255) ? rel_o : 255;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        uint32_t w = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) w |= (uint32_t)lane_gather(v, 16 * q + 4 * i + g) << (8 * i);
        ob[q] = w;
    }
}
// the same through 64 bytes of LDS: row r files its byte at (r % 4) * 16 + r / 4, so that the sixteen
// bytes a lane group needs are one 16-byte read
__device__ __forceinline__ void orow_to_operand_bytes_lds(char *lds_idx, int rel_o, int lane, uint32_t (&ob)[4]) {
    const int g = lane >> 4;
    const int v = (rel_o >= 0 && rel_o < 255) ? rel_o : 255;
    reinterpret_cast<unsigned char *>(lds_idx)[(lane & 3) * 16 + (lane >> 2)] = (unsigned char)v;
    wave_lds_fence();
    const uint4 w = *reinterpret_cast<const uint4 *>(lds_idx + 16 * g);
    ob[0] = w.x; ob[1] = w.y; ob[2] = w.z; ob[3] = w.w;
    wave_lds_fence();
}

// For T consecutive tiles of sixteen output rows, t = 0..T-1:  D[t][j][i] += sum over rows of
// [index byte of row == 16 t + 4 (lane / 16) + i] * x[row][8c + j];  Dn[t][i] += number of such rows.  Rows in
// registers, on v_mfma_f32_16x16x32_bf16 (contraction step qq covers rows 32 qq .. 32 qq + 31; index
// (lane / 16, i), i = 0..7, stands for row 32 qq + 4 i + lane / 16 = register 8 qq + i): the B operand is built once
// per column group and shared by the tiles.  Index bytes are relative to the first of the T tiles.
template <int T>
__device__ __forceinline__ void membership_mfma_tiles(const RowRegs &x, const uint32_t (&ob)[4], int c, int q_hi,
                                                      floatx4_t (&D)[T][8], floatx4_t (&Dn)[T]) {
    const uint4 ones = make_uint4(0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u);
#pragma unroll
    for (int qq = 0; qq < 2; ++qq) {
        if (2 * qq < q_hi) {
            bf16x8f_t a[T];
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const uint32_t want = (uint32_t)(c + 16 * t);
                uint32_t aw[4];
#pragma unroll
                for (int h2 = 0; h2 < 2; ++h2) {
                    const uint32_t b4 = ob[2 * qq + h2];
                    const uint32_t m0 = (((b4 >> 0) & 0xFFu) == want) ? 0x3F80u : 0u;
                    const uint32_t m1 = (((b4 >> 8) & 0xFFu) == want) ? 0x3F80u : 0u;
                    const uint32_t m2 = (((b4 >> 16) & 0xFFu) == want) ? 0x3F80u : 0u;
                    const uint32_t m3 = (((b4 >> 24) & 0xFFu) == want) ? 0x3F80u : 0u;
                    aw[2 * h2] = m0 | (m1 << 16);
                    aw[2 * h2 + 1] = m2 | (m3 << 16);
                }
                a[t] = __builtin_bit_cast(bf16x8f_t, make_uint4(aw[0], aw[1], aw[2], aw[3]));
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                uint32_t w[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const uint32_t d0 = dword_of(x.r[8 * qq + 2 * k], j >> 1), d1 = dword_of(x.r[8 * qq + 2 * k + 1], j >> 1);
                    w[k] = (j & 1) ? pack_hi(d0, d1) : pack_lo(d0, d1);
                }
                const bf16x8f_t bop = __builtin_bit_cast(bf16x8f_t, make_uint4(w[0], w[1], w[2], w[3]));
#pragma unroll
                for (int t = 0; t < T; ++t) D[t][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[t], bop, D[t][j], 0, 0, 0);
            }
#pragma unroll
            for (int t = 0; t < T; ++t) Dn[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[t], __builtin_bit_cast(bf16x8f_t, ones), Dn[t], 0, 0, 0);
        }
    }
}

// keys and values of a window in one sweep: the keys come back from the LDS copy made by gram_bitmatrix
// (32 rows at a time), the values are in registers; both share the 0/1 operand.  v_mfma_f32_16x16x32_bf16:
// contraction step qq covers rows 32 qq .. 32 qq + 31, its index (lane / 16, i), i = 0..7, stands for row
// 32 qq + 4 i + lane / 16 = register 8 qq + i of the lane's own group.
__device__ __forceinline__ void membership_mfma_kv(const char *lds, const RowRegs &xv, const uint32_t (&ob)[4], int want,
                                                   int q_hi, int lane, floatx4_t (&DK)[8], floatx4_t (&DV)[8], floatx4_t &Dn) {
    const int g = lane >> 4, c = lane & 15;
    const uint4 ones = make_uint4(0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u);
#pragma unroll
    for (int qq = 0; qq < 2; ++qq) {
        if (2 * qq < q_hi) {
            uint4 r[8];
#pragma unroll
            for (int i = 0; i < 8; ++i)
                r[i] = *reinterpret_cast<const uint4 *>(lds + (4 * (8 * qq + i) + g) * kLdsRowBytes + 16 * c);
            uint32_t aw[4];
#pragma unroll
            for (int h2 = 0; h2 < 2; ++h2) {
                const uint32_t b4 = ob[2 * qq + h2];
                const uint32_t m0 = (((b4 >> 0) & 0xFFu) == (uint32_t)want) ? 0x3F80u : 0u;
                const uint32_t m1 = (((b4 >> 8) & 0xFFu) == (uint32_t)want) ? 0x3F80u : 0u;
                const uint32_t m2 = (((b4 >> 16) & 0xFFu) == (uint32_t)want) ? 0x3F80u : 0u;
                const uint32_t m3 = (((b4 >> 24) & 0xFFu) == (uint32_t)want) ? 0x3F80u : 0u;
                aw[2 * h2] = m0 | (m1 << 16);
                aw[2 * h2 + 1] = m2 | (m3 << 16);
            }
            const bf16x8f_t a = __builtin_bit_cast(bf16x8f_t, make_uint4(aw[0], aw[1], aw[2], aw[3]));
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                {
                    uint32_t w[4];
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        const uint32_t d0 = dword_of(r[2 * t], j >> 1), d1 = dword_of(r[2 * t + 1], j >> 1);
                        w[t] = (j & 1) ? pack_hi(d0, d1) : pack_lo(d0, d1);
                    }
                    DK[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8f_t, make_uint4(w[0], w[1], w[2], w[3])), DK[j], 0, 0, 0);
                }
                {
                    uint32_t w[4];
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        const uint32_t d0 = dword_of(xv.r[8 * qq + 2 * t], j >> 1), d1 = dword_of(xv.r[8 * qq + 2 * t + 1], j >> 1);
                        w[t] = (j & 1) ? pack_hi(d0, d1) : pack_lo(d0, d1);
                    }
                    DV[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8f_t, make_uint4(w[0], w[1], w[2], w[3])), DV[j], 0, 0, 0);
                }
            }
            Dn = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8f_t, ones), Dn, 0, 0, 0);
        }
    }
}

// ------------------------------------------------------------------------------------------------
// All pairwise similarities of a window at once (Eq. 2 for every pair the seeds of Alg. 1 can ask for).
// The window's rows are parked in LDS (row stride 272 B) and read back in the operand layout of
// v_mfma_f32_16x16x32_bf16 (lane l: row l%16 of a 16-row tile, elements 8*(l/16)..+7 of a 32-element
// slice); a tile of keys is both the A operand (rows m) and the B operand (rows n) of the Gram tile
// G[m][n] = k_m . k_n.  The ten upper-triangle tiles of the 64 x 64 Gram matrix take 40 MFMAs.
// Each lane then turns its 4 x 10 dot products into cosines, compares them with tau and files the
// outcome as bit m of a per-column word; an OR over the four lane groups completes the words, and lane
// r (row order) ends up with  yes[r]: bit m set iff Sim(m, r) > tau + band   (m < r or same tile)
//                             unsure[r]: bit m set iff the fp32 value is within the band (or not a number).
__device__ __forceinline__ uint32_t or_rows(uint32_t x) {   // OR over the four 16-lane rows, same lane position
    auto r = __builtin_amdgcn_permlane16_swap(x, x, false, false);
    x = r[0] | r[1];
    r = __builtin_amdgcn_permlane32_swap(x, x, false, false);
    return r[0] | r[1];
}

// Gram tiles (I, J), I <= J < NT, of the rows parked in LDS; tile k = index in the 4 x 4 upper triangle
template <int NT>
__device__ __forceinline__ void gram_tiles(const char *lds, int g, int c, floatx4_t (&acc)[10]) {
    // v_mfma_f32_16x16x32_bf16: 32 elements of the contraction per product (lane l: elements 8 * (l / 16) .. + 7
    // of a 32-element slice), the form that runs at the full bf16 rate of this chip
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        bf16x8f_t a[NT];
#pragma unroll
        for (int I = 0; I < NT; ++I) {
            const uint4 v = *reinterpret_cast<const uint4 *>(lds + (16 * I + c) * kLdsRowBytes + (32 * ks + 8 * g) * 2);
            a[I] = __builtin_bit_cast(bf16x8f_t, v);
        }
#pragma unroll
        for (int I = 0; I < NT; ++I)
#pragma unroll
            for (int J = I; J < NT; ++J) {
                constexpr int base[4] = {0, 4, 7, 9};
                const int k = base[I] + (J - I);
                acc[k] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[I], a[J], acc[k], 0, 0, 0);
            }
    }
}

// Outcome for lane r (row order):  yes_row: bit m set iff Sim(m, r) > tau + band (for m < r, and for the
// m > r of r's own 16-row tile);  unsure_row: bit m set iff the fp32 value lies within the band or a
// norm is unusable.  The common case (no pair of the window anywhere near tau) never builds the
// unsure words: every lane tracks the smallest distance to tau it has seen instead.
__device__ __forceinline__ void gram_bitmatrix(char *lds, const RowRegs &x, int R, float tau, int lane,
                                               uint64_t &yes_row, uint64_t &unsure_row) {
    const int g = lane >> 4, c = lane & 15;
    float *s_rinv = reinterpret_cast<float *>(lds + kLdsRinvOff);
    uint32_t *s_bits = reinterpret_cast<uint32_t *>(lds + kLdsBitsOff);
#pragma unroll
    for (int t = 0; t < 16; ++t)
        *reinterpret_cast<uint4 *>(lds + (4 * t + g) * kLdsRowBytes + 16 * c) = x.r[t];
    *reinterpret_cast<uint4 *>(s_bits + 4 * lane) = make_uint4(0u, 0u, 0u, 0u);
    wave_lds_fence();

    const int nt = (R + 15) >> 4;   // 16-row tiles in use
    floatx4_t acc[10];
#pragma unroll
    for (int k = 0; k < 10; ++k) acc[k] = floatx4_t{0.f, 0.f, 0.f, 0.f};
    if (nt >= 4) gram_tiles<4>(lds, g, c, acc);
    else if (nt == 3) gram_tiles<3>(lds, g, c, acc);
    else if (nt == 2) gram_tiles<2>(lds, g, c, acc);
    else gram_tiles<1>(lds, g, c, acc);
    // squared norms are the diagonal of the Gram matrix: tile (I, I), row 4g+i == column c
    {
        const int kd[4] = {0, 4, 7, 9};
#pragma unroll
        for (int I = 0; I < 4; ++I) {
            const int i = c - 4 * g;
            const floatx4_t d = acc[kd[I]];
            const float nsq = (i == 0) ? d[0] : ((i == 1) ? d[1] : ((i == 2) ? d[2] : d[3]));
            if (i >= 0 && i < 4) s_rinv[16 * I + c] = safe_rinv(nsq);
        }
    }
    wave_lds_fence();
    // sim(m, n) > t  <=>  dot * rinv_m > t * norm_n.  Per pair one fused multiply-add gives
    //     dd = (tau + band) * norm_n - dot * rinv_m :   dd < 0  the pair is above the band (a sure yes),
    //     0 <= dd <= 2 * band * norm_n  inside the band (unsure),  beyond that a sure no;
    // its sign bit is shifted into a nibble (v_alignbit), and an unsigned minimum over the bit patterns
    // keeps the smallest non-negative dd the lane has seen (negative values compare as huge).
    float hn[4], wn[4];
    floatx4_t rm[4];
    bool bad = false;
#pragma unroll
    for (int I = 0; I < 4; ++I) {
        const float rn = s_rinv[16 * I + c];
        const float norm = __builtin_amdgcn_rcpf(rn);
        bad = bad || (16 * I + c < R && !(rn == rn));
        hn[I] = (tau + kFastBand) * norm;
        wn[I] = (2.0f * kFastBand) * norm;
        rm[I] = *reinterpret_cast<const floatx4_t *>(s_rinv + 16 * I + 4 * g);
    }
    // per column tile J: bits m (0..63) as two dwords (row 16*I + 4g + i at bit 16*(I&1) + 4g + i of word I>>1)
    uint32_t y[4][2];
    uint32_t dmin[4];
#pragma unroll
    for (int J = 0; J < 4; ++J) { y[J][0] = y[J][1] = 0u; dmin[J] = 0x7F800000u; }
    {
        constexpr int base[4] = {0, 4, 7, 9};
#pragma unroll
        for (int I = 0; I < 4; ++I)
#pragma unroll
            for (int J = I; J < 4; ++J) {
                if (J < nt) {
                    const int k = base[I] + (J - I);
                    uint32_t nib = 0u;
#pragma unroll
                    for (int i = 3; i >= 0; --i) {
                        const uint32_t dd = __float_as_uint(fmaf(-acc[k][i], rm[I][i], hn[J]));
                        nib = __builtin_amdgcn_alignbit(nib, dd, 31);     // (nib << 1) | sign bit
                        dmin[J] = min(dmin[J], dd);
                    }
                    y[J][I >> 1] |= nib << (16 * (I & 1) + 4 * g);
                }
            }
    }
    // complete the words over the four lane groups; lane r = 16J + c keeps the words of its own row
    uint32_t yl = 0u, yh = 0u;
#pragma unroll
    for (int J = 0; J < 4; ++J) {
        if (J < nt) {
            const uint32_t a0 = or_rows(y[J][0]);
            const uint32_t a1 = (nt > 2) ? or_rows(y[J][1]) : 0u;   // rows 32.. exist only then
            if (g == J) { yl = a0; yh = a1; }
        }
    }
    // anything close to tau, or an unusable norm, anywhere in the window?  (rare)
    bool close = bad;
#pragma unroll
    for (int J = 0; J < 4; ++J) close = close || (J < nt && dmin[J] <= __float_as_uint(wn[J]));
    if (ballot64(close) != 0ull) {
        // the same products and bounds as above, so that "yes", "no" and "unsure" partition the pairs
        constexpr int base[4] = {0, 4, 7, 9};
#pragma unroll
        for (int J = 0; J < 4; ++J) {
            uint32_t u0 = 0u, u1 = 0u;
#pragma unroll
            for (int I = 0; I <= J; ++I) {
                if (J < nt) {
                    const int k = base[I] + (J - I);
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float dd = fmaf(-acc[k][i], rm[I][i], hn[J]);
                        const bool uu = !(dd < 0.f) && !(dd > wn[J]);     // also true for a value that is not a number
                        const uint32_t bit = 1u << (16 * (I & 1) + 4 * g + i);
                        if (I < 2) u0 |= uu ? bit : 0u; else u1 |= uu ? bit : 0u;
                    }
                }
            }
            if (J < nt) {
                __hip_atomic_fetch_or(s_bits + 4 * (16 * J + c) + 2, u0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                __hip_atomic_fetch_or(s_bits + 4 * (16 * J + c) + 3, u1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
        }
        wave_lds_fence();
        const uint2 w = *reinterpret_cast<const uint2 *>(s_bits + 4 * lane + 2);
        unsure_row = ((uint64_t)w.y << 32) | w.x;
    } else {
        unsure_row = 0ull;
    }
    // a pair that is unsure must not also count as a sure yes
    yes_row = (((uint64_t)yh << 32) | yl) & ~unsure_row;
    wave_lds_fence();   // the LDS area is reused by the next window
}

__device__ __forceinline__ bool cosine_exceeds_f64_lds(const char *lds, int row_a, int row_b, float tau, int lane) {
    double dot = 0.0, ss = 0.0, cc = 0.0;
#pragma unroll
    for (int k = 0; k < kFastD / kWave; ++k) {
        const int e = (lane & (kWave - 1)) + k * kWave;
        const double a = load1_f64(reinterpret_cast<const bf16_t *>(lds + row_a * kLdsRowBytes) + e);
        const double b = load1_f64(reinterpret_cast<const bf16_t *>(lds + row_b * kLdsRowBytes) + e);
        dot += a * b; ss += a * a; cc += b * b;
    }
    dot = wave_allreduce_sum(dot);
    ss = wave_allreduce_sum(ss);
    cc = wave_allreduce_sum(cc);
    return dot / (sqrt(ss) * sqrt(cc)) > (double)tau;   // NaN compares false
}

// Alg. 1 over the open rows of a window or block without walking the seeds one by one.  Seeds are taken in row
// order and a seed absorbs every open row of its chunk that resembles it, so a row joins the FIRST seed before
// it that it resembles and is a seed itself iff there is none: the seed set T is the one set with
//     r in T  <=>  no row of T before r (in r's chunk) resembles r            (induction over r: unique).
// With F(S) = { r : no row of S before r resembles r }, T is the only fixed point of F.  Starting from the rows
// that nothing earlier resembles (all of them seeds), F is applied until the set stops changing; when
// "resembles" is transitive inside the chunks, the usual case, that is the first application.  Lane r brings,
// restricted to the open rows before r in its own chunk, the rows it surely resembles (ye) and those inside
// the band around tau (ue).  A pair inside the band can change the outcome only if its earlier row is a seed
// that the later row, a seed itself, might resemble after all, or one before the seed the later row joins: the
// first such pair of every row is settled in fp64 (the keys are parked in LDS) and the fixed point is taken
// again.  Returns false, with nothing decided, if the set has not settled after a few applications of F or
// pairs keep turning up: the caller then takes the seeds one at a time.
__device__ __forceinline__ bool first_fit_fixed_point(const char *lds, uint64_t ye, uint64_t ue, bool is_open, float tau, int lane,
                                                      uint64_t &seeds, int &my_seed) {
    for (int pass = 0; pass < 8; ++pass) {
        uint64_t S = ballot64(is_open && ye == 0ull);
        bool settled = false;
        for (int it = 0; it < 8 && !settled; ++it) {
            const uint64_t S2 = ballot64(is_open && (ye & S) == 0ull);
            settled = S2 == S;
            S = S2;
        }
        if (!settled) return false;
        const bool is_seed = (S >> lane) & 1ull;
        const uint64_t mine = ye & S;                                   // not empty unless the row is a seed
        const int first = is_seed ? lane : first_bit(mine);
        const uint64_t doubt = ue & S & (is_seed ? ~0ull : bits_below(first & 63));
        uint64_t doubtful = ballot64(is_open && doubt != 0ull);
        if (doubtful == 0ull) {
            seeds = S;
            my_seed = is_open ? first : -1;
            return true;
        }
        const int sd_mine = first_bit(doubt);
        while (doubtful != 0ull) {
            const int j = first_bit(doubtful);
            doubtful &= doubtful - 1ull;
            const int sd = __builtin_amdgcn_readlane(sd_mine, j);
            const bool res = cosine_exceeds_f64_lds(lds, sd, j, tau, lane);
            if (lane == j) {
                ue &= ~(1ull << sd);
                if (res) ye |= 1ull << sd;
            }
        }
    }
    return false;
}

__device__ __forceinline__ int nth_set_bit(uint64_t m, int k) {   // position of the k-th set bit, 0 <= k < popcount(m)
    int pos = 0;
#pragma unroll
    for (int w = 32; w >= 1; w >>= 1) {
        const uint64_t part = (m >> pos) & ((1ull << w) - 1ull);
        const int cnt = __popcll(part);
        if (k >= cnt) { k -= cnt; pos += w; }
    }
    return pos;
}

// ------------------------------------------------------------------------------------------------
// Work decomposition shared by both passes: a task is `chunks_per_item` (<= 32) consecutive chunks of
// one (sequence, head), handled by one single-wavefront workgroup, so a finished task frees its
// registers and LDS at once and the hardware dispatcher balances the load.  The task's chunk offsets
// live in one register (lane j holds offsets[m0 + j]) and are read with v_readlane.
struct TaskOffsets {
    int v;      // lane j: offsets[m0 + j] for j <= nch
    int m0, M;
    __device__ __forceinline__ int at(int j) const { return __builtin_amdgcn_readlane(v, j); }
    // rows of chunk idx of the task including its closing delimiter (the last chunk of a sequence has none)
    __device__ __forceinline__ int rows(int idx) const {
        return (m0 + idx < M - 1) ? (at(idx + 1) - at(idx)) : (at(idx + 1) - 1 - at(idx));
    }
};

constexpr int kFastTaskThreads = kWave;

// ------------------------------------------------------------------------------------------------
// store the sizes of tile `ot` (from the ones column) at provisional rows
__device__ __forceinline__ void store_sizes(const floatx4_t &Dn, int ot, int n_out, int32_t *dst, int64_t dst_row0,
                                            int64_t row_limit, int lane) {
    if ((lane & 15) == 0) {
        const int g = lane >> 4;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int o = 16 * ot + 4 * g + i;
            if (o < n_out && dst_row0 + o < row_limit) dst[dst_row0 + o] = (int)(Dn[i] + 0.5f);
        }
    }
}

template <typename TO>
__global__ __launch_bounds__(kFastTaskThreads, 2) void gsc_compress_kernel(GscParams p) {
    __shared__ __attribute__((aligned(16))) char s_lds[kLdsWaveBytes];
    // One-dimensional grid: workgroup id = (pass * grid_x + x) * (B * Hkv) + (sequence, head).  The
    // workgroups of pass 0 are dispatched first and take the tasks that need more than one window, pass 1
    // takes the rest, so the long tasks never start last.  Inside a pass the task index x varies slowest:
    // the workgroups beyond a sequence's last task (the host cannot know how many chunks there are) then
    // come in one burst at the end of the pass instead of between the heads.
    const int n_bh_grid = p.B * p.Hkv;
    const int per_pass = p.grid_x * n_bh_grid;
    const int pass = (int)blockIdx.x / per_pass;
    const int rem_id = (int)blockIdx.x - pass * per_pass;
    const int wg_x = rem_id / n_bh_grid, bh_id = rem_id - wg_x * n_bh_grid;
    const int b = bh_id / p.Hkv, h = bh_id - b * p.Hkv;
    const int lane_id = threadIdx.x;
    const int C = p.chunks_per_item;
    // The offsets of the workgroup's first task are requested together with the chunk count instead of
    // after it (which offsets are meaningful is decided once the count is known; the index is clamped to
    // the row, so the early request is always inside the array).  Most workgroups only look at one task,
    // many only to find that it belongs to the other pass: for them this halves the time to the exit.
    const int32_t *off = p.offsets + (int64_t)b * p.offsets_stride_b;
    const int first_v = (lane_id <= C) ? off[min((int64_t)wg_x * C + lane_id, p.offsets_stride_b - 1)] : 0;
    const int M = __builtin_amdgcn_readfirstlane(p.num_chunks[b]);
    if (M <= 0) return;
    int n = p.seq_lens ? __builtin_amdgcn_readfirstlane(p.seq_lens[b]) : p.N_max;
    n = n < 0 ? 0 : (n > p.N_max ? p.N_max : n);
    const int tasks = (M + C - 1) / C;
    const int64_t bh = (int64_t)b * p.Hkv + h;
    const bf16_t *Kbh = reinterpret_cast<const bf16_t *>(p.K) + b * p.stride_b + h * p.stride_h;
    const bf16_t *Vbh = reinterpret_cast<const bf16_t *>(p.V) + b * p.stride_b + h * p.stride_h;
    int32_t *pcount_bh = p.pcount + bh * ((int64_t)p.N_max + 1);
    int32_t *seed_bh = p.seedrow + bh * p.N_max;
    int32_t *cid_bh = p.cluster_id ? p.cluster_id + bh * p.N_max : nullptr;   // only when the caller asked
    int32_t *cid32_bh = p.cid + bh * p.N_max;                                    // always there (workspace)
    int32_t *stmp_bh = p.stmp + bh * p.N_max;
    TO *ktmp_c = reinterpret_cast<TO *>(p.ktmp) + bh * (int64_t)p.N_max * kFastD;
    TO *vtmp_c = reinterpret_cast<TO *>(p.vtmp) + bh * (int64_t)p.N_max * kFastD;
    const int64_t tmp_rows = p.N_max;
    const float tau = p.tau_dev ? *p.tau_dev : p.tau;
    const bool count_only = p.count_only != 0;

    for (int task = wg_x; task < tasks; task += p.grid_x) {
        TaskOffsets to;
        to.m0 = task * C;
        to.M = M;
        const int m0 = to.m0;
        const int nch = min(C, M - m0);
        if (task == wg_x) to.v = (lane_id <= nch) ? first_v : 0;
        else to.v = (lane_id <= nch) ? off[m0 + lane_id] : 0;
        {
            const int task_rows = to.at(nch) - to.at(0) - ((m0 + nch == M) ? 1 : 0);
            if ((task_rows > kWin) != (pass == 0)) continue;
        }
        int idx = 0;
        while (idx < nch) {
            // Everything derived from the lane number is recomputed per window (and per block of a long
            // chunk) instead of being carried in registers across the whole kernel: the optimiser cannot
            // see through the empty asm statement.
            int lane = lane_id;
            asm volatile("" : "+v"(lane));
            const int g = lane >> 4, c = lane & 15;
            const int rows_first = to.rows(idx);
            const int w0 = to.at(idx);
            if (rows_first <= kWin) {
                // ---------------- window of whole chunks, at most 64 rows
                int idx_hi = idx, R = 0;
                while (idx_hi < nch) {
                    const int rr = to.rows(idx_hi);
                    if (R + rr > kWin) break;
                    R += rr;
                    idx_hi += 1;
                }
                const int nchw = idx_hi - idx;
                RowRegs xk, xv;
                load_rows(xk, row_source(Kbh, p.stride_n, w0, R, g, c));
                // the values are not needed before the merge: requested now, they arrive under the Gram step
                // (a counting call reads none: the descriptor is empty and the loads come back as zeros)
                load_rows(xv, row_source(Vbh, p.stride_n, w0, count_only ? 0 : R, g, c));
                // chunk range [lo, hi) of every row; a delimiter is a one-row range of its own
                int lo = lane, hi = lane + 1;
                bool in_chunk = false;
                for (int j = 0; j < nchw; ++j) {
                    const int cs = to.at(idx + j) - w0;
                    const int ce = to.at(idx + j + 1) - 1 - w0;
                    if (lane >= cs && lane < ce) { lo = cs; hi = ce; in_chunk = true; }
                }
                uint64_t yes_row, unsure_row;
                gram_bitmatrix(s_lds, xk, R, tau, lane, yes_row, unsure_row);
                // Alg. 1 on the bit matrix, one seed per chunk and round: the first unassigned row of a
                // chunk is its next seed and absorbs the unassigned rows of the chunk whose bit is set
                const uint64_t my_range = bits_range(lo, hi);
                uint64_t todo = bits_range(0, R);
                uint64_t seedmask = 0ull;
                int my_seed = -1;
                {
                    const uint64_t earlier = bits_below(lane) & my_range;
                    if (first_fit_fixed_point(s_lds, yes_row & earlier, unsure_row & earlier, lane < R, tau, lane, seedmask, my_seed)) todo = 0ull;
                }
                while (todo != 0ull) {
                    const uint64_t mine = todo & my_range;
                    const int s = (mine != 0ull) ? (__ffsll((unsigned long long)mine) - 1) : 64;
                    const bool open = (todo >> lane) & 1ull;
                    const bool is_seed = open && (s == lane);
                    const bool cand = open && (s != lane);
                    bool yes = cand && ((yes_row >> (s & 63)) & 1ull);
                    uint64_t recheck = ballot64(cand && ((unsure_row >> (s & 63)) & 1ull));
                    while (recheck != 0ull) {
                        const int j = __builtin_amdgcn_readfirstlane(first_bit(recheck));
                        recheck &= recheck - 1ull;
                        const int sj = __builtin_amdgcn_readlane(s, j);
                        const bool res = cosine_exceeds_f64_lds(s_lds, sj, j, tau, lane);
                        if (lane == j) yes = res;
                    }
                    const uint64_t seeds_now = ballot64(is_seed);
                    const uint64_t got = ballot64(yes);
                    if (is_seed || yes) my_seed = s;
                    seedmask |= seeds_now;
                    todo &= ~(seeds_now | got);
                }
                // seeds in row order are the output rows of the window
                const int nseed = __popcll(seedmask);
                const int my_o = (lane < R) ? __popcll(seedmask & bits_range(0, my_seed)) : -1;
                if (cid_bh && lane < R)
                    cid_bh[w0 + lane] = in_chunk ? __popcll(seedmask & bits_range(lo, my_seed)) : -1;
                {
                    const int cs = __shfl(to.v, min(idx + lane, 63), kWave) - w0;
                    const int ce = __shfl(to.v, min(idx + lane + 1, 63), kWave) - 1 - w0;
                    if (lane < nchw) pcount_bh[m0 + idx + lane] = __popcll(seedmask & bits_range(cs, ce));
                }
                // cluster means -> provisional rows [w0, w0 + nseed): keys (back from LDS), then values
                uint32_t ob[4];
                orow_to_operand_bytes_lds(s_lds + kLdsIdxOff, my_o, lane, ob);
                const int q_hi = (R + 15) >> 4;
                for (int ot = 0; ot * 16 < nseed && !count_only; ++ot) {
                    floatx4_t DK[8], DV[8], Dn = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int j = 0; j < 8; ++j) DK[j] = DV[j] = Dn;
                    membership_mfma_kv(s_lds, xv, ob, 16 * ot + c, q_hi, lane, DK, DV, Dn);
                    store_tile<TO>(DK, Dn, ot, nseed, ktmp_c, (int64_t)w0, tmp_rows, lane);
                    store_tile<TO>(DV, Dn, ot, nseed, vtmp_c, (int64_t)w0, tmp_rows, lane);
                    store_sizes(Dn, ot, nseed, stmp_bh, (int64_t)w0, tmp_rows, lane);
                }
                idx = idx_hi;
            } else {
                // ---------------- one chunk longer than a window: one sweep over blocks of 64 rows.
                // The first sixteen clusters live in registers across the blocks: their seeds' keys as the
                // A operand of a (seed x row) Gram product, their key/value sums as MFMA accumulators.
                // Clusters beyond the sixteenth (rare) take the slow way: seed by seed against the block,
                // and a second pass over the chunk per sixteen further output rows.
                const int start = w0;
                const int l = to.at(idx + 1) - 1 - start;
                const bool closed = (start + l) < n;
                int nseeds = 0;
                uint4 sa[4];   // lane (c, g): elements 32 ks + 8 g .. + 7 of the key of seed c (the MFMA's A operand)
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) sa[ks] = make_uint4(0u, 0u, 0u, 0u);
                floatx4_t DK[8], DV[8], Dn = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int j = 0; j < 8; ++j) DK[j] = DV[j] = Dn;
                float *s_rinv = reinterpret_cast<float *>(s_lds + kLdsRinvOff);
                float *s_seed_rinv = reinterpret_cast<float *>(s_lds + kLdsSeedRinvOff);
                for (int rb = 0; rb < l; rb += kWin) {
                    int lane = lane_id;
                    asm volatile("" : "+v"(lane));
                    const int g = lane >> 4, c = lane & 15;
                    const int R = min(kWin, l - rb);
                    const int nt = (R + 15) >> 4;
                    const bf16_t *block0 = Kbh + (int64_t)(start + rb) * p.stride_n;
                    uint64_t yes_row, unsure_row;
                    {
                        RowRegs x;
                        load_rows(x, row_source(Kbh, p.stride_n, start + rb, R, g, c));
                        gram_bitmatrix(s_lds, x, R, tau, lane, yes_row, unsure_row);
                    }
                    RowRegs xv;
                    load_rows(xv, row_source(Vbh, p.stride_n, start + rb, count_only ? 0 : R, g, c));
                    uint64_t todo = bits_range(0, R);
                    int my_o = -1;
                    const int seeds_before = nseeds;
                    // carried seeds, sixteen at a time: their similarities with every row of the block are one
                    // (seed x row) Gram product; the first group's keys sit in registers, further groups
                    // (rare) are fetched again
                    for (int sg = 0; sg * 16 < seeds_before && todo != 0ull; ++sg) {
                        const int ns = min(16, seeds_before - 16 * sg);
                        uint4 sb[4];
                        floatx4_t rs;
                        if (sg == 0) {
#pragma unroll
                            for (int ks = 0; ks < 4; ++ks) sb[ks] = sa[ks];
                            rs = *reinterpret_cast<const floatx4_t *>(s_seed_rinv + 4 * g);
                        } else {
                            const int srow_c = (c < ns) ? __hip_atomic_load(seed_bh + start + 16 * sg + c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0;
                            const bf16_t *sp = Kbh + (int64_t)(start + srow_c) * p.stride_n + 8 * g;
#pragma unroll
                            for (int ks = 0; ks < 4; ++ks)
                                sb[ks] = (c < ns) ? *reinterpret_cast<const uint4 *>(sp + 32 * ks) : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                const int sl = 16 * sg + 4 * g + i;
                                rs[i] = (4 * g + i < ns) ? __int_as_float(__hip_atomic_load(stmp_bh + start + sl, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) : 0.f;
                            }
                        }
                        // (seed x row) products: lane (c, g) gets seeds 4g .. 4g+3 against row 16 J + c
                        floatx4_t cx[4];
#pragma unroll
                        for (int J = 0; J < 4; ++J) cx[J] = floatx4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int ks = 0; ks < 4; ++ks) {
                            const bf16x8f_t a = __builtin_bit_cast(bf16x8f_t, sb[ks]);
#pragma unroll
                            for (int J = 0; J < 4; ++J) {
                                if (J < nt) {
                                    const uint4 v = *reinterpret_cast<const uint4 *>(s_lds + (16 * J + c) * kLdsRowBytes + (32 * ks + 8 * g) * 2);
                                    cx[J] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8f_t, v), cx[J], 0, 0, 0);
                                }
                            }
                        }
                        // per row one word: bit s = surely similar to seed s of the group, bit 16 + s = inside the
                        // band.  A lane has the bits of its four seeds; an OR over the four lane groups completes
                        // the word of row 16 J + c, and lane r keeps the word of row r.
                        uint32_t cw = 0u;
#pragma unroll
                        for (int J = 0; J < 4; ++J) {
                            if (J < nt) {
                                const float norm = __builtin_amdgcn_rcpf(s_rinv[16 * J + c]);
                                const float hn = (tau + kFastBand) * norm, ln = (tau - kFastBand) * norm;
                                uint32_t w = 0u;
#pragma unroll
                                for (int i = 0; i < 4; ++i) {
                                    const float t = cx[J][i] * rs[i];
                                    const bool yy = t > hn;
                                    const bool uu = !yy && !(t < ln);
                                    w |= (yy ? 1u : 0u) << (4 * g + i);
                                    w |= (uu ? 1u : 0u) << (16 + 4 * g + i);
                                }
                                w = or_rows(w);
                                if (g == J) cw = w;
                            }
                        }
                        const uint32_t valid = (1u << ns) - 1u;
                        const bool open = (todo >> lane) & 1ull;
                        uint32_t cyes = open ? (cw & valid) : 0u;
                        uint32_t cuns = open ? ((cw >> 16) & valid) : 0u;
                        // first fit over the seeds of the group; a pair inside the band is settled in fp64
                        // when it is the first candidate of its row
                        for (;;) {
                            const uint32_t pend = cyes | cuns;
                            const int f = (pend != 0u) ? (__ffs(pend) - 1) : -1;
                            const uint64_t need = ballot64(f >= 0 && ((cuns >> (f & 31)) & 1u));
                            if (need == 0ull) break;
                            const int j = __builtin_amdgcn_readfirstlane(first_bit(need));
                            const int fj = __builtin_amdgcn_readlane(f, j);
                            const int srow = __hip_atomic_load(seed_bh + start + 16 * sg + fj, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            const bool res = cosine_exceeds_f64_fast(Kbh + (int64_t)(start + srow) * p.stride_n,
                                                                     block0 + (int64_t)j * p.stride_n, tau, lane);
                            if (lane == j) {
                                cuns &= ~(1u << fj);
                                if (res) cyes |= 1u << fj;
                            }
                        }
                        if (cyes != 0u) my_o = 16 * sg + __ffs(cyes) - 1;
                        todo &= ~ballot64(cyes != 0u);
                    }
                    // seeds inside the block, from the bit matrix
                    // (the rows still open are decided among themselves; the new seeds continue the chunk's numbering)
                    int new_row = -1;   // lane (c, g): block row of the seed that takes register slot c in this block
                    uint64_t new_seeds = 0ull;
                    {
                        const uint64_t earlier_open = bits_below(lane) & todo;
                        const bool is_open = (todo >> lane) & 1ull;
                        uint64_t S = 0ull;
                        int my_seed = -1;
                        if (first_fit_fixed_point(s_lds, yes_row & earlier_open, unsure_row & earlier_open, is_open, tau, lane, S, my_seed)) {
                            if (is_open) my_o = nseeds + __popcll(S & bits_below(my_seed));
                            const int k = c - nseeds;
                            if (k >= 0 && k < (int)__popcll(S)) new_row = nth_set_bit(S, k);
                            new_seeds = S;
                            nseeds += __popcll(S);
                            todo = 0ull;
                        }
                    }
                    while (todo != 0ull) {
                        const int i = __builtin_amdgcn_readfirstlane(first_bit(todo));
                        todo &= ~(1ull << i);
                        new_seeds |= 1ull << i;
                        const int o = nseeds;
                        nseeds += 1;
                        if (o < 16 && c == o) new_row = i;
                        const bool cand = (todo >> lane) & 1ull;
                        bool yes = cand && ((yes_row >> i) & 1ull);
                        uint64_t recheck = ballot64(cand && ((unsure_row >> i) & 1ull));
                        while (recheck != 0ull) {
                            const int j = __builtin_amdgcn_readfirstlane(first_bit(recheck));
                            recheck &= recheck - 1ull;
                            const bool res = cosine_exceeds_f64_lds(s_lds, i, j, tau, lane);
                            if (lane == j) yes = res;
                        }
                        const uint64_t got = ballot64(yes);
                        todo &= ~got;
                        if (lane == i || yes) my_o = o;
                    }
                    // seed list of the chunk, filed by the new seeds themselves once the block is decided: row,
                    // and reciprocal norm (in the size staging area, which gets its final contents only after
                    // the last block)
                    if ((new_seeds >> lane) & 1ull) {
                        const float ri = s_rinv[lane];
                        if (my_o < 16) s_seed_rinv[my_o] = ri;
                        __hip_atomic_store(seed_bh + start + my_o, rb + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        __hip_atomic_store(stmp_bh + start + my_o, __float_as_int(ri), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                    // new seeds move into their register slots (keys still parked in LDS)
                    if (ballot64(new_row >= 0) != 0ull) {
#pragma unroll
                        for (int ks = 0; ks < 4; ++ks) {
                            const uint4 v = *reinterpret_cast<const uint4 *>(s_lds + max(new_row, 0) * kLdsRowBytes + (32 * ks + 8 * g) * 2);
                            if (new_row >= 0) sa[ks] = v;
                        }
                    }
                    // cluster index of every row: the caller's output, and what the passes for clusters
                    // beyond the sixteenth read back below (through L2, by this wave only)
                    if (lane < R) __hip_atomic_store(cid32_bh + start + rb + lane, my_o, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    // sums of the first sixteen clusters
                    uint32_t ob[4];
                    orow_to_operand_bytes_lds(s_lds + kLdsIdxOff, (lane < R) ? my_o : -1, lane, ob);
                    if (!count_only) membership_mfma_kv(s_lds, xv, ob, c, nt, lane, DK, DV, Dn);
                    wave_lds_fence();   // the next block overwrites the parked keys and the seed tables are read above
                }
                if (closed && lane == 0 && cid_bh) cid_bh[start + l] = -1;
                if (lane == 0) pcount_bh[m0 + idx] = nseeds;
                if (count_only) {
                    idx += 1;
                    continue;
                }
                {
                    const int n0 = min(nseeds, 16);
                    store_tile<TO>(DK, Dn, 0, n0, ktmp_c, (int64_t)start, tmp_rows, lane);
                    store_tile<TO>(DV, Dn, 0, n0, vtmp_c, (int64_t)start, tmp_rows, lane);
                    store_sizes(Dn, 0, n0, stmp_bh, (int64_t)start, tmp_rows, lane);
                }
                if (nseeds > 16) {
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");   // cluster index stores are done
                    // kExtraTiles tiles of sixteen clusters per sweep over the chunk, keys and values in sweeps
                    // of their own (the accumulators of both, or of a third tile, would not fit the registers).
                    // The read-once hint stays on these loads: without it the large configurations lose more
                    // to the displaced provisional rows than the sweeps gain from finding their rows cached.
                    constexpr int kExtraTiles = 2;
                    for (int src = 0; src < 2; ++src) {
                        const bf16_t *Xbh = (src == 0) ? Kbh : Vbh;
                        TO *dst_c = (src == 0) ? ktmp_c : vtmp_c;
                        for (int ot = 1; ot * 16 < nseeds; ot += kExtraTiles) {
                            floatx4_t D[kExtraTiles][8], Dm[kExtraTiles];
#pragma unroll
                            for (int t = 0; t < kExtraTiles; ++t) {
                                Dm[t] = floatx4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                                for (int j = 0; j < 8; ++j) D[t][j] = Dm[t];
                            }
                            for (int rb = 0; rb < l; rb += kWin) {
                                const int R = min(kWin, l - rb);
                                RowRegs x;
                                load_rows(x, row_source(Xbh, p.stride_n, start + rb, R, g, c));
                                int my_o = -1;
                                if (lane < R)
                                    my_o = __hip_atomic_load(cid32_bh + start + rb + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                                uint32_t ob[4];
                                orow_to_operand_bytes(my_o - 16 * ot, lane, ob);
                                membership_mfma_tiles<kExtraTiles>(x, ob, c, (R + 15) >> 4, D, Dm);
                            }
#pragma unroll
                            for (int t = 0; t < kExtraTiles; ++t) {
                                if ((ot + t) * 16 < nseeds) {
                                    store_tile<TO>(D[t], Dm[t], ot + t, nseeds, dst_c, (int64_t)start, tmp_rows, lane);
                                    if (src == 1) store_sizes(Dm[t], ot + t, nseeds, stmp_bh, (int64_t)start, tmp_rows, lane);
                                }
                            }
                        }
                    }
                }
                if (closed && start + nseeds < tmp_rows) {
                    // the closing delimiter is output row `nseeds`: a copy with size 1
                    if (g == 0) {
                        float kv[8], vv[8];
                        load8(Kbh + (int64_t)(start + l) * p.stride_n + 8 * c, kv);
                        load8(Vbh + (int64_t)(start + l) * p.stride_n + 8 * c, vv);
                        store8(ktmp_c + (int64_t)(start + nseeds) * kFastD + 8 * c, kv);
                        store8(vtmp_c + (int64_t)(start + nseeds) * kFastD + 8 * c, vv);
                    }
                    if (lane == 0) stmp_bh[start + nseeds] = 1;
                }
                idx += 1;
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Moves merged rows from their provisional position (first rows of their window / long chunk) to
// their final position rowbase[first chunk] + o.  Pure copy: 16 lanes per row, four rows per access.
// INLINE_PREFIX: no scan kernel ran; every workgroup adds up the cluster counts of the chunks before
// its task itself (a few KB from L2), and the workgroup of the last task files the total.  Worth it
// while a sequence has a few thousand chunks: it saves a launch whose only job is that sum.
// APPEND: the rows go behind the base_lens[b, h] rows the outputs already hold (with the scan kernel in
// between, its row bases already include them).
template <typename TO, bool INLINE_PREFIX, bool APPEND>
__global__ __launch_bounds__(kFastTaskThreads) void gsc_relocate_kernel(GscParams p) {
    // one-dimensional grid, task index slowest (see the compress kernel)
    const int n_bh_grid = p.B * p.Hkv;
    const int wg_x = (int)blockIdx.x / n_bh_grid, bh_id = (int)blockIdx.x - wg_x * n_bh_grid;
    const int b = bh_id / p.Hkv, h = bh_id - b * p.Hkv;
    const int lane = threadIdx.x;
    const int g = lane >> 4, c = lane & 15;
    const int C = p.chunks_per_item;
    const int32_t *off = p.offsets + (int64_t)b * p.offsets_stride_b;
    // offsets of the first task requested together with the chunk count (index clamped to the row)
    const int first_v = (lane <= C) ? off[min((int64_t)wg_x * C + lane, p.offsets_stride_b - 1)] : 0;
    const int M = __builtin_amdgcn_readfirstlane(p.num_chunks[b]);
    const int64_t bh = (int64_t)b * p.Hkv + h;
    if (M <= 0) {
        if (INLINE_PREFIX && wg_x == 0 && lane == 0) p.comp_lens[bh] = -1;
        return;
    }
    const int tasks = (M + C - 1) / C;
    const int32_t *rowbase_bh = p.rowbase + bh * ((int64_t)p.N_max + 2);
    const int32_t *pcount_bh = p.pcount + bh * ((int64_t)p.N_max + 1);
    const int32_t *stmp_bh = p.stmp + bh * p.N_max;
    const TO *ktmp_c = reinterpret_cast<const TO *>(p.ktmp) + bh * (int64_t)p.N_max * kFastD + 8 * c;
    const TO *vtmp_c = reinterpret_cast<const TO *>(p.vtmp) + bh * (int64_t)p.N_max * kFastD + 8 * c;
    TO *Kc_c = reinterpret_cast<TO *>(p.Kc) + bh * (int64_t)p.cap * kFastD + 8 * c;
    TO *Vc_c = reinterpret_cast<TO *>(p.Vc) + bh * (int64_t)p.cap * kFastD + 8 * c;
    int32_t *counts_bh = p.counts + bh * p.cap;
    const int64_t cap = p.cap;
    constexpr int NP = (int)sizeof(TO) * 8 / 16;   // 16-byte pieces per lane and row
    bool base_bad = false;
    const int base_rows = (INLINE_PREFIX && APPEND) ? gsc_base_rows(p, bh, base_bad) : 0;

    int summed = 0, summed_to = 0;      // INLINE_PREFIX: cluster counts of the chunks [0, summed_to), added up
    for (int task = wg_x; task < tasks; task += p.grid_x) {
        TaskOffsets to;
        to.m0 = task * C;
        to.M = M;
        const int m0 = to.m0;
        const int nch = min(C, M - m0);
        if (task == wg_x) to.v = (lane <= nch) ? first_v : 0;
        else to.v = (lane <= nch) ? off[m0 + lane] : 0;
        int basev;
        if (INLINE_PREFIX) {
            // rows of the chunks before the task: every one of them is closed by a delimiter
            // 2048 counts per round, four per lane and load, through a descriptor that ends at the task's first
            // chunk (what lies beyond reads as zero): all loads of a round are in flight together, and a
            // sequence of up to 32k tokens with chunks of 16 rows or more needs one round
            // A workgroup that takes several tasks (more tasks than workgroups: very short chunks) carries the
            // sum on from its previous task instead of starting at the first chunk again.
            const __amdgpu_buffer_rsrc_t pc_src = __builtin_amdgcn_make_buffer_rsrc(const_cast<int32_t *>(pcount_bh + summed_to), (short)0,
                                                                                    (m0 - summed_to) * 4, 0x00020000);
            const int mine_raw = (lane < nch) ? pcount_bh[m0 + lane] : 0;
            int part = 0;
            for (int mb = 0; mb < m0 - summed_to; mb += 32 * kWave) {
                u32x4_t t[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) t[j] = __builtin_amdgcn_raw_buffer_load_b128(pc_src, (mb + 4 * kWave * j + 4 * lane) * 4, 0, 0);
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    part += (int)(((t[j].x & kPcountMask) + (t[j].y & kPcountMask)) + ((t[j].z & kPcountMask) + (t[j].w & kPcountMask)));
            }
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) part += __shfl_xor(part, d, kWave);
            summed += part;
            summed_to = m0;
            const int before = summed;
            // lane j: first output row of chunk m0 + j (lane nch: one past the task)
            int mine = (lane < nch) ? (mine_raw & kPcountMask) + ((m0 + lane < M - 1) ? 1 : 0) : 0;
            int incl = mine;
#pragma unroll
            for (int d = 1; d < kWave; d <<= 1) {
                const int up = __shfl_up(incl, d, kWave);
                if (lane >= d) incl += up;
            }
            basev = base_rows + before + m0 + incl - mine;
            if (m0 + nch == M && lane == nch) p.comp_lens[bh] = (!base_bad && basev <= p.cap) ? basev : -1;
        } else {
            basev = (lane <= nch) ? rowbase_bh[m0 + lane] : 0;
        }
        int idx = 0;
        while (idx < nch) {
            const int src0 = to.at(idx);
            const int64_t out0 = __builtin_amdgcn_readlane(basev, idx);
            int idx_hi = idx + 1;
            if (to.rows(idx) <= kWin) {
                int R = 0;
                idx_hi = idx;
                while (idx_hi < nch) {
                    const int rr = to.rows(idx_hi);
                    if (R + rr > kWin) break;
                    R += rr;
                    idx_hi += 1;
                }
            }
            const int n_out = __builtin_amdgcn_readlane(basev, idx_hi) - (int)out0;
            for (int o0 = 0; o0 < n_out; o0 += 16) {
                uint4 kk[4][NP], vv[4][NP];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int o = o0 + 4 * k + g;
                    const bool ok = o < n_out && out0 + o < cap;
                    const uint4 *ks = reinterpret_cast<const uint4 *>(ktmp_c + ((int64_t)src0 + (ok ? o : 0)) * kFastD);
                    const uint4 *vs = reinterpret_cast<const uint4 *>(vtmp_c + ((int64_t)src0 + (ok ? o : 0)) * kFastD);
#pragma unroll
                    for (int q = 0; q < NP; ++q) {
                        kk[k][q] = ok ? load16_stream(ks + q) : make_uint4(0, 0, 0, 0);
                        vv[k][q] = ok ? load16_stream(vs + q) : make_uint4(0, 0, 0, 0);
                    }
                }
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int o = o0 + 4 * k + g;
                    if (o < n_out && out0 + o < cap) {
                        uint4 *kd = reinterpret_cast<uint4 *>(Kc_c + (out0 + o) * kFastD);
                        uint4 *vd = reinterpret_cast<uint4 *>(Vc_c + (out0 + o) * kFastD);
#pragma unroll
                        for (int q = 0; q < NP; ++q) { store16_stream(kd + q, kk[k][q]); store16_stream(vd + q, vv[k][q]); }
                    }
                }
            }
            for (int o = lane; o < n_out; o += kWave)
                if (out0 + o < cap) counts_bh[out0 + o] = stmp_bh[src0 + o];
            idx = idx_hi;
        }
    }
}

// ------------------------------------------------------------------------------------------------
hipError_t launch_gsc_fast(const GscParams &p, hipStream_t stream) {
    // Single-wave workgroups, each looping over the tasks x, x + grid_x, ... of its (sequence, head).  A
    // workgroup that takes one task is faster than one that walks several, and the host cannot know how many
    // tasks there are: with chunks of a few dozen tokens, about one per 21 tokens per chunk of the task.  A
    // small call gets a workgroup per expected task; a large one, where the many workgroups that find no task
    // (a microsecond of one wave slot each) would cost more than the walking, one per two.  Shorter chunks
    // make the workgroups loop, longer ones leave more of them without a task.
    const int max_tasks = (p.N_max + 1 + p.chunks_per_item - 1) / p.chunks_per_item;
    int gx = tuning().gsc_grid_x;
    if (gx <= 0) {
        const int64_t rows_in_call = (int64_t)p.B * p.Hkv * p.N_max;
        const int tokens_per_wg = 21 * p.chunks_per_item * (rows_in_call <= (int64_t(1) << 19) ? 1 : 2);
        gx = max(16, p.N_max / tokens_per_wg);
    }
    gx = max(1, min(max_tasks, gx));
    GscParams pc = p;
    pc.grid_x = gx;
    const dim3 grid2((unsigned)(2 * gx * p.Hkv * p.B));   // two passes over the tasks: long ones first
    const dim3 grid1((unsigned)(gx * p.Hkv * p.B));
    if (p.out_is_bf16) hipLaunchKernelGGL((gsc_compress_kernel<bf16_t>), grid2, dim3(kFastTaskThreads), 0, stream, pc);
    else hipLaunchKernelGGL((gsc_compress_kernel<float>), grid2, dim3(kFastTaskThreads), 0, stream, pc);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (p.count_only) return launch_gsc_scan(p, stream);   // adds up the counts: comp_lens, and nothing else is wanted
    // Up to 32k tokens the relocation adds up the cluster counts before its task itself (one round of loads
    // per 2048 chunks; a sequence that is all delimiters costs sixteen rounds per workgroup, 0.8 ms per call);
    // longer sequences get the scan kernel, which does the sum once per (sequence, head) whatever the
    // number of chunks.
    const bool inline_prefix = p.N_max <= 32768;
    if (!inline_prefix) {
        e = launch_gsc_scan(p, stream);
        if (e != hipSuccess) return e;
    }
    {
        if (inline_prefix) {
            if (p.base_lens) {
                if (p.out_is_bf16) hipLaunchKernelGGL((gsc_relocate_kernel<bf16_t, true, true>), grid1, dim3(kFastTaskThreads), 0, stream, pc);
                else hipLaunchKernelGGL((gsc_relocate_kernel<float, true, true>), grid1, dim3(kFastTaskThreads), 0, stream, pc);
            } else {
                if (p.out_is_bf16) hipLaunchKernelGGL((gsc_relocate_kernel<bf16_t, true, false>), grid1, dim3(kFastTaskThreads), 0, stream, pc);
                else hipLaunchKernelGGL((gsc_relocate_kernel<float, true, false>), grid1, dim3(kFastTaskThreads), 0, stream, pc);
            }
        } else {
            if (p.out_is_bf16) hipLaunchKernelGGL((gsc_relocate_kernel<bf16_t, false, false>), grid1, dim3(kFastTaskThreads), 0, stream, pc);
            else hipLaunchKernelGGL((gsc_relocate_kernel<float, false, false>), grid1, dim3(kFastTaskThreads), 0, stream, pc);
        }
        e = hipGetLastError();
    }
    return e;
}

}  // namespace sc
