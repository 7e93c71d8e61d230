// sc_segment: delimiter mask -> chunk offsets (paper Sec. 2.2, Eq. 1).
//
// One workgroup of 1024 threads per 32 KiB of a sequence's mask: every thread reads 32 mask bytes with two
// 16-byte loads (both in flight together, requested together with the sequence length, not after it), turns
// them into a 32-bit "is delimiter" word, a block-wide exclusive scan of the popcounts gives each thread the
// rank of its first delimiter, and the positions are scattered to offsets[rank + 1].  Pure integer work; a
// sequence of up to 32k tokens is one workgroup and HBM traffic the mask once.
#include "sc_device.h"
#include "sc_host.h"

namespace sc {

constexpr int kSegThreads = 1024;
constexpr int kSegBytesPerThread = 32;

__device__ __forceinline__ uint32_t nonzero_bytes4(uint32_t w) {
    // bit k set iff byte k of w is nonzero
    uint32_t r = 0;
    r |= (w & 0x000000ffu) ? 1u : 0u;
    r |= (w & 0x0000ff00u) ? 2u : 0u;
    r |= (w & 0x00ff0000u) ? 4u : 0u;
    r |= (w & 0xff000000u) ? 8u : 0u;
    return r;
}

// delimiter bits of the 32 mask bytes of a thread that start at byte i0 of a row (bytes at and beyond n dropped)
__device__ __forceinline__ uint32_t delimiter_bits32(const uint8_t *row, int i0, int n, int n_max, bool aligned) {
    // (whether the 32 bytes may be read depends on the row's capacity, not on the sequence length: the
    // request does not wait for seq_lens[b])
    if (i0 + kSegBytesPerThread <= n_max && aligned) {
        const uint4 v0 = *reinterpret_cast<const uint4 *>(row + i0), v1 = *reinterpret_cast<const uint4 *>(row + i0 + 16);
        const uint32_t lo = nonzero_bytes4(v0.x) | (nonzero_bytes4(v0.y) << 4) | (nonzero_bytes4(v0.z) << 8) | (nonzero_bytes4(v0.w) << 12);
        const uint32_t hi = nonzero_bytes4(v1.x) | (nonzero_bytes4(v1.y) << 4) | (nonzero_bytes4(v1.z) << 8) | (nonzero_bytes4(v1.w) << 12);
        const uint32_t x = lo | (hi << 16);
        const int keep = n - i0;   // bytes of this thread inside the sequence
        return (keep >= kSegBytesPerThread) ? x : ((keep <= 0) ? 0u : (x & ((1u << keep) - 1u)));
    }
    uint32_t x = 0;
    for (int k = 0; k < kSegBytesPerThread; ++k)
        if (i0 + k < n && row[i0 + k] != 0) x |= 1u << k;
    return x;
}

// Workgroup (t, b) files the delimiters of tile t (32 KiB of mask) of sequence b.  Their ranks start at the
// number of delimiters in the tiles before, which the workgroup counts itself (reading those tiles again, all
// requests in flight together) instead of waiting for its neighbours: no workgroup depends on another, and
// a 131 072-token sequence takes one trip to memory on four compute units instead of four in a row on one.
__global__ __launch_bounds__(kSegThreads) void segment_kernel(
    const uint8_t *__restrict__ mask, int64_t mask_stride_b, const int32_t *__restrict__ seq_lens, int n_max,
    int32_t *__restrict__ offsets, int64_t offsets_stride_b, int offsets_cap, int32_t *__restrict__ num_chunks) {
    __shared__ int s_wave_total[kSegThreads / kWave];
    __shared__ int s_wave_before[kSegThreads / kWave];
    __shared__ int s_tile_total, s_before_total;
    constexpr int kTile = kSegThreads * kSegBytesPerThread;

    const int b = blockIdx.x, t = blockIdx.y;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid / kWave;
    int n = seq_lens ? seq_lens[b] : n_max;
    n = n < 0 ? 0 : (n > n_max ? n_max : n);
    const uint8_t *row = mask + (int64_t)b * mask_stride_b;
    int32_t *off = offsets + (int64_t)b * offsets_stride_b;
    const bool aligned = ((reinterpret_cast<uintptr_t>(row) & 15u) == 0);
    const bool last_tile = t == (int)gridDim.y - 1;

    if (t == 0 && tid == 0) off[0] = 0;
    // delimiters in the tiles before this one (this thread's share), then this tile's own
    int before = 0;
    for (int j = 0; j < t; ++j) before += __popc(delimiter_bits32(row, j * kTile + tid * kSegBytesPerThread, n, n_max, aligned));
    const int i0 = t * kTile + tid * kSegBytesPerThread;
    uint32_t bits = delimiter_bits32(row, i0, n, n_max, aligned);
    const int cnt = __popc(bits);
    // inclusive scan inside the wave (own tile), sum over the wave (tiles before)
    int incl = cnt, bsum = before;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const int up = __shfl_up(incl, d, kWave);
        if (lane >= d) incl += up;
        bsum += __shfl_xor(bsum, d, kWave);
    }
    if (lane == kWave - 1) s_wave_total[wave] = incl;
    if (lane == 0) s_wave_before[wave] = bsum;
    __syncthreads();
    if (wave == 0) {
        int v = (lane < kSegThreads / kWave) ? s_wave_total[lane] : 0;
        int vb = (lane < kSegThreads / kWave) ? s_wave_before[lane] : 0;
        int ti = v;
#pragma unroll
        for (int d = 1; d < kSegThreads / kWave; d <<= 1) {
            const int up = __shfl_up(ti, d, kWave);
            if (lane >= d) ti += up;
            vb += __shfl_xor(vb, d, kWave);
        }
        if (lane < kSegThreads / kWave) s_wave_total[lane] = ti - v;  // exclusive wave prefix
        if (lane == kSegThreads / kWave - 1) s_tile_total = ti;
        if (lane == 0) s_before_total = vb;
    }
    __syncthreads();
    const int running = s_before_total;
    int rank = running + s_wave_total[wave] + incl - cnt;  // delimiters before this thread's bytes
    while (bits) {
        const int k = __ffs((int)bits) - 1;
        bits &= bits - 1;
        rank += 1;
        if (rank < offsets_cap) off[rank] = i0 + k + 1;
    }
    if (last_tile && tid == 0) {
        const int M = running + s_tile_total + 1;
        if (M + 1 <= offsets_cap) {
            off[M] = n + 1;
            num_chunks[b] = M;
        } else {
            num_chunks[b] = -1;
        }
    }
}

hipError_t launch_segment(const uint8_t *mask, int64_t mask_stride_b, const int32_t *seq_lens, int B, int n_max,
                          int32_t *offsets, int64_t offsets_stride_b, int offsets_cap, int32_t *num_chunks,
                          hipStream_t stream) {
    const int tiles = (n_max + kSegThreads * kSegBytesPerThread - 1) / (kSegThreads * kSegBytesPerThread);
    hipLaunchKernelGGL(segment_kernel, dim3(B, tiles), dim3(kSegThreads), 0, stream, mask, mask_stride_b, seq_lens, n_max,
                       offsets, offsets_stride_b, offsets_cap, num_chunks);
    return hipGetLastError();
}

}  // namespace sc
