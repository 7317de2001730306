// Kernels and helpers the two GPU-side encoders (ecf8_encode.hip, ecfw_encode.hip) share.
#ifndef ECF8_ENC_DEVICE_H
#define ECF8_ENC_DEVICE_H

#include "ecf8_device.h"

namespace {

__global__ __launch_bounds__(256) void fill_zero_kernel(uint64_t dst, uint64_t bytes)   // bytes % 16 == 0
{
    GLOBAL u32x4 *p = (GLOBAL u32x4 *)dst;
    const uint64_t n16 = bytes / 16;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (uint64_t)gridDim.x * blockDim.x)
        p[i] = u32x4{0, 0, 0, 0};
}

// In-place inclusive prefix sum of chunk_bit[1 .. n_chunks] (chunk_bit[0] = 0): one workgroup.
__global__ __launch_bounds__(1024) void scan_kernel(uint64_t chunk_bit_, uint64_t n_chunks)
{
    __shared__ uint64_t wave_sum[16];
    __shared__ uint64_t carry_s;
    GLOBAL uint64_t *cb = (GLOBAL uint64_t *)chunk_bit_;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) carry_s = 0;
    __syncthreads();
    for (uint64_t base = 1; base <= n_chunks; base += 1024) {
        const uint64_t i = base + tid;
        uint64_t v = i <= n_chunks ? cb[i] : 0;
        // inclusive scan inside the wave (values < 2^32 per chunk, sums in 64 bits)
        for (int d = 1; d < 64; d <<= 1) {
            const uint64_t up = __shfl_up(v, d, 64);
            if (lane >= d) v += up;
        }
        if (lane == 63) wave_sum[wave] = v;
        __syncthreads();
        uint64_t before = carry_s;
        for (int w = 0; w < wave; w++) before += wave_sum[w];
        if (i <= n_chunks) cb[i] = v + before;
        __syncthreads();
        if (tid == 1023) carry_s = v + before;
        __syncthreads();
    }
}

int grid_for_bytes(uint64_t work_items, int per_block)
{
    int cus = device_cus();
    if (cus <= 0) return -1;
    uint64_t want = (work_items + per_block - 1) / per_block;
    uint64_t cap = (uint64_t)cus * 8;
    uint64_t g = want < cap ? want : cap;
    return (int)(g ? g : 1);
}


} // namespace

#endif
