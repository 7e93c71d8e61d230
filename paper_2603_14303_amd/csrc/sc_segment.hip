// sc_segment: delimiter mask -> chunk offsets (paper Sec. 2.2, Eq. 1).
//
// One workgroup of 1024 threads walks one sequence in tiles of 32 KiB of mask: every thread reads
// 32 mask bytes with two 16-byte loads (both in flight together), turns them into a 64-bit "is
// delimiter" word, a block-wide exclusive scan of the popcounts gives each thread the rank of its first
// delimiter, and the positions are scattered to offsets[rank + 1].  A tile costs three barriers, so a
// 32k-token sequence is one tile.  The mask bytes of the first tile are requested together with the sequence
// length, not after it.  Pure integer work, HBM traffic = the mask once.
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

__global__ __launch_bounds__(kSegThreads) void segment_kernel(
    const uint8_t *__restrict__ mask, int64_t mask_stride_b, const int32_t *__restrict__ seq_lens, int n_max,
    int32_t *__restrict__ offsets, int64_t offsets_stride_b, int offsets_cap, int32_t *__restrict__ num_chunks) {
    __shared__ int s_wave_total[kSegThreads / kWave];
    __shared__ int s_tile_total;

    const int b = blockIdx.x;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid / kWave;
    int n = seq_lens ? seq_lens[b] : n_max;
    n = n < 0 ? 0 : (n > n_max ? n_max : n);
    const uint8_t *row = mask + (int64_t)b * mask_stride_b;
    int32_t *off = offsets + (int64_t)b * offsets_stride_b;
    const bool aligned = ((reinterpret_cast<uintptr_t>(row) & 15u) == 0);

    if (tid == 0) off[0] = 0;
    int running = 0;  // delimiters found in earlier tiles
    // (the first tile always runs, so that its requests are issued before the length is known; an empty
    // sequence finds no delimiter in it)
    int base = 0;
    do {
        const int i0 = base + tid * kSegBytesPerThread;
        uint64_t bits = 0;
        // (whether the 32 bytes may be read depends on the row's capacity, not on the sequence length: the
        // request does not wait for seq_lens[b]; bytes at and beyond the length are dropped afterwards)
        if (i0 + kSegBytesPerThread <= n_max && aligned) {
            constexpr int kLoads = kSegBytesPerThread / 16;
            uint4 v[kLoads];
#pragma unroll
            for (int q = 0; q < kLoads; ++q) v[q] = *reinterpret_cast<const uint4 *>(row + i0 + 16 * q);
#pragma unroll
            for (int q = 0; q < kLoads; ++q) {
                const uint32_t b16 = nonzero_bytes4(v[q].x) | (nonzero_bytes4(v[q].y) << 4) | (nonzero_bytes4(v[q].z) << 8) |
                                     (nonzero_bytes4(v[q].w) << 12);
                bits |= (uint64_t)b16 << (16 * q);
            }
            const int keep = n - i0;   // bytes of this thread inside the sequence
            bits = (keep >= kSegBytesPerThread) ? bits : ((keep <= 0) ? 0ull : (bits & ((1ull << keep) - 1ull)));
        } else {
            for (int k = 0; k < kSegBytesPerThread; ++k)
                if (i0 + k < n && row[i0 + k] != 0) bits |= 1ull << k;
        }
        const int cnt = __popcll(bits);
        // inclusive scan inside the wave
        int incl = cnt;
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            const int up = __shfl_up(incl, d, kWave);
            if (lane >= d) incl += up;
        }
        if (lane == kWave - 1) s_wave_total[wave] = incl;
        __syncthreads();
        if (wave == 0) {
            int t = (lane < kSegThreads / kWave) ? s_wave_total[lane] : 0;
            int ti = t;
#pragma unroll
            for (int d = 1; d < kSegThreads / kWave; d <<= 1) {
                const int up = __shfl_up(ti, d, kWave);
                if (lane >= d) ti += up;
            }
            if (lane < kSegThreads / kWave) s_wave_total[lane] = ti - t;  // exclusive wave prefix
            if (lane == kSegThreads / kWave - 1) s_tile_total = ti;
        }
        __syncthreads();
        int rank = running + s_wave_total[wave] + incl - cnt;  // delimiters before this thread's bytes
        const int tile_total = s_tile_total;
        while (bits) {
            const int k = __ffsll((unsigned long long)bits) - 1;
            bits &= bits - 1;
            rank += 1;
            if (rank < offsets_cap) off[rank] = i0 + k + 1;
        }
        running += tile_total;
        __syncthreads();  // s_wave_total / s_tile_total are reused by the next tile
        base += kSegThreads * kSegBytesPerThread;
    } while (base < n);
    if (tid == 0) {
        const int M = running + 1;
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
    hipLaunchKernelGGL(segment_kernel, dim3(B), dim3(kSegThreads), 0, stream, mask, mask_stride_b, seq_lens, n_max,
                       offsets, offsets_stride_b, offsets_cap, num_chunks);
    return hipGetLastError();
}

}  // namespace sc
