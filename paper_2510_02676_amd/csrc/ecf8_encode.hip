// GPU-side ECF8 encoder for gfx950 (paper Section 3.1: histogram, code, stream, metadata and
// nibble plane, produced on the device so that FP8 checkpoints compress at load time without a
// trip through host memory).  Writes exactly the container the CPU encoder writes, byte for
// byte: the code and the layout come from the same host routine, fed with the device histogram.
//
//   fill 0 -> histogram (LDS counters private to each thread, 16 atomics per workgroup)
//   -> [host: 128 bytes back, code + layout]
//   -> fill 0, header (+ pair table built in LDS) -> lane_bits and chunk totals (one wave per
//   chunk) -> prefix sum of the totals (one workgroup) -> stream (one wave per chunk assembles
//   its span in LDS with ds_or, copies it out; the two dwords a span may share with its
//   neighbours go out with atomic OR) -> nibble plane (one dword per 8 elements).
// No scratch memory: the histogram is counted into the header's freq[] field and the chunk
// totals into chunk_bit[], both part of the output.
#include "ecf8_device.h"
#include "ecf8_enc_device.h"
#include "ecf8_plan.h"

namespace {

struct EncArgs {
    uint64_t x, blob;                     // device addresses
    uint64_t n, cols, n_chunks;
    uint64_t off_cb, off_lb, off_st, off_pl, st_bytes;
    uint32_t N, group, tiled;
    uint64_t len_packed;                  // code length of symbol s in bits 4s..4s+3
    uint32_t code[16], rcode[16];
};

// element index of the 16-element piece q of lane l of chunk c (see the container's layouts)
__device__ __forceinline__ uint64_t piece_start(const EncArgs &a, uint64_t c, uint32_t l, uint32_t q)
{
    const uint64_t E = 64ull * a.N;
    if (a.tiled) {
        const uint64_t kc_per_row = a.cols / (4ull * a.N);
        return ((c / kc_per_row) * 16 + (l & 15)) * a.cols + (c % kc_per_row) * (4ull * a.N) + 64ull * q + 16ull * (l >> 4);
    }
    const uint64_t grouped = (a.n / E) & ~((uint64_t)a.group - 1);
    if (c < grouped) {
        const uint64_t w = c & (a.group - 1);
        return (c - w) * E + w * 1024 + (uint64_t)q * a.group * 1024 + l * 16ull;
    }
    return c * E + q * 1024ull + l * 16ull;
}

// Exponent-field histogram into 16 u64 counters.  Every thread counts into its own 16 LDS words
// (bank = thread, no conflicts, no atomics); one atomic add per bin per workgroup at the end.
__global__ __launch_bounds__(256) void histogram_kernel(uint64_t x_, uint64_t n, uint64_t counters_)
{
    __shared__ uint32_t cnt[16 * 256];
    const GLOBAL uint8_t *x = (const GLOBAL uint8_t *)x_;
    GLOBAL unsigned long long *counters = (GLOBAL unsigned long long *)counters_;
    const int tid = threadIdx.x;
    for (int s = 0; s < 16; s++) cnt[s * 256 + tid] = 0;
    const uint64_t n16 = n / 16;
    for (uint64_t i = (uint64_t)blockIdx.x * 256 + tid; i < n16; i += (uint64_t)gridDim.x * 256) {
        const u32x4 v = __builtin_nontemporal_load((const GLOBAL u32x4 *)x + i);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int k = 0; k < 4; k++)
#pragma unroll
            for (int b = 0; b < 4; b++) cnt[((w[k] >> (8 * b + 3)) & 15u) * 256 + tid]++;
    }
    if (blockIdx.x == 0)
        for (uint64_t i = n16 * 16 + tid; i < n; i += 256) cnt[((x[i] >> 3) & 15u) * 256 + tid]++;
    __syncthreads();
    if (tid < 16) {
        unsigned long long sum = 0;
        for (int t = 0; t < 256; t++) sum += cnt[tid * 256 + ((t + tid) & 255)];
        if (sum) atomicAdd((unsigned long long *)(counters + tid), sum);
    }
}

// Header, and the decoder's pair table built with the kernels' own builder.
__global__ __launch_bounds__(1024) void header_kernel(uint64_t blob_, ecf8_header h)
{
    __shared__ __attribute__((aligned(16))) uint8_t smem[4 * TBL_ENTRIES + 128];
    GLOBAL uint8_t *blob = (GLOBAL uint8_t *)blob_;
    const int tid = threadIdx.x;
    if (tid < 64) ((GLOBAL uint32_t *)blob)[tid] = ((const uint32_t *)&h)[tid];
    if (h.table_bits) {
        uint16_t *tbl = (uint16_t *)smem;
        uint32_t *s_len = (uint32_t *)(smem + 4 * TBL_ENTRIES);
        uint64_t len_lo, len_hi;
        __builtin_memcpy(&len_lo, h.code_len, 8);
        __builtin_memcpy(&len_hi, h.code_len + 8, 8);
        build_tables(len_lo, len_hi, tbl, s_len, s_len + 16, (uint16_t *)(smem + 2 * TBL_ENTRIES), tid, 1024);
        for (int i = tid; i < TBL_ENTRIES * 2 / 16; i += 1024) ((GLOBAL u32x4 *)(blob + 256))[i] = ((const u32x4 *)tbl)[i];
    }
}

// lane_bits[c][l] = code bits of the lane's symbols; chunk_bit[c + 1] = bits of chunk c
// (turned into stream positions by the scan below).  One wave per chunk.
__global__ __launch_bounds__(256) void lane_bits_kernel(EncArgs a)
{
    const int lane = threadIdx.x & 63;
    const uint64_t c = (uint64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (c >= a.n_chunks) return;
    const GLOBAL uint8_t *x = (const GLOBAL uint8_t *)a.x;
    uint32_t lb = 0;
    for (uint32_t q = 0; q < a.N / 16; q++) {
        const uint64_t e = piece_start(a, c, lane, q);
        if (e + 16 <= a.n) {
            const u32x4 v = *(const GLOBAL u32x4 *)(x + e);
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int k = 0; k < 4; k++)
#pragma unroll
                for (int b = 0; b < 4; b++) lb += (uint32_t)(a.len_packed >> (4 * ((w[k] >> (8 * b + 3)) & 15u))) & 15u;
        } else {
            for (uint64_t i = e; i < a.n && i < e + 16; i++) lb += (uint32_t)(a.len_packed >> (4 * ((x[i] >> 3) & 15u))) & 15u;
        }
    }
    ((GLOBAL uint16_t *)(a.blob + a.off_lb))[c * 64 + lane] = (uint16_t)lb;
    const uint32_t total = wave_incl_scan(lb);
    if (lane == 63) ((GLOBAL uint64_t *)(a.blob + a.off_cb))[c + 1] = total;
}

// Stream: one wave per chunk.  The span's dwords are assembled in LDS (every lane ORs its
// codewords in: forward run up from its first bit, backward run down from its last), then copied
// out; the first and the last dword of a span can hold bits of neighbouring chunks and go out
// with atomic OR onto the zeroed stream.
template <int STAGE_DWORDS>
__global__ __launch_bounds__(256) void pack_kernel(EncArgs a)
{
    __shared__ uint32_t stage_all[4][STAGE_DWORDS];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t c = (uint64_t)blockIdx.x * 4 + wave;
    if (c >= a.n_chunks) return;
    uint32_t *stage = stage_all[wave];
    const GLOBAL uint8_t *x = (const GLOBAL uint8_t *)a.x;
    const GLOBAL uint64_t *cb = (const GLOBAL uint64_t *)(a.blob + a.off_cb);
    const uint64_t b0 = cb[c], b1 = cb[c + 1];
    const uint32_t lb = ((const GLOBAL uint16_t *)(a.blob + a.off_lb))[c * 64 + lane];
    const uint64_t first_dw = b0 >> 5, end_dw = (b1 + 31) >> 5;      // dwords [first_dw, end_dw) hold the span
    const uint32_t n_dw = (uint32_t)(end_dw - first_dw);
    for (uint32_t i = lane; i < n_dw && i < (uint32_t)STAGE_DWORDS; i += 64) stage[i] = 0;
    __builtin_amdgcn_wave_barrier();
    uint32_t fwd = (uint32_t)(b0 & 31) + (wave_incl_scan(lb) - lb);  // stage bit of the lane's first bit
    uint32_t bwd = fwd + lb;                                         // one past its last bit
    auto put = [&](uint32_t at, uint32_t bits, uint32_t nb) {
        const uint32_t d = at >> 5, sh = at & 31;
        __hip_atomic_fetch_or(&stage[d], bits << sh, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        if (sh + nb > 32) __hip_atomic_fetch_or(&stage[d + 1], bits >> (32 - sh), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    };
    const uint32_t P = a.N / 16;
    for (uint32_t q = 0; q < P; q++) {
        const uint64_t e = piece_start(a, c, lane, q);
        for (uint32_t j = 0; j < 16 && e + j < a.n; j++) {
            const uint32_t s = (x[e + j] >> 3) & 15u;
            const uint32_t l = (uint32_t)(a.len_packed >> (4 * s)) & 15u;
            if (q < P / 2) { put(fwd, a.rcode[s], l); fwd += l; }
            else { bwd -= l; put(bwd, a.code[s], l); }
        }
    }
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
    GLOBAL uint32_t *out = (GLOBAL uint32_t *)(a.blob + a.off_st);
    for (uint32_t i = lane; i < n_dw; i += 64) {
        const uint32_t v = stage[i];
        if (i == 0 || i + 1 == n_dw) { if (v) atomicOr((unsigned int *)(out + first_dw + i), v); }
        else out[first_dw + i] = v;
    }
}

// Nibble plane: 8 elements -> 4 bytes (byte j: low nibble element j, high nibble element j + 4).
__global__ __launch_bounds__(256) void plane_kernel(EncArgs a)
{
    const GLOBAL uint8_t *x = (const GLOBAL uint8_t *)a.x;
    GLOBAL uint32_t *plane = (GLOBAL uint32_t *)(a.blob + a.off_pl);
    const uint64_t groups = (a.n + 7) / 8;
    for (uint64_t g = (uint64_t)blockIdx.x * 256 + threadIdx.x; g < groups; g += (uint64_t)gridDim.x * 256) {
        uint32_t lo = 0, hi = 0;
        if (g * 8 + 8 <= a.n) {
            const u32x2 v = *(const GLOBAL u32x2 *)(x + g * 8);
            lo = v.x;
            hi = v.y;
        } else {
            for (uint64_t i = g * 8; i < a.n; i++) {
                const uint32_t j = (uint32_t)(i - g * 8);
                if (j < 4) lo |= (uint32_t)x[i] << (8 * j); else hi |= (uint32_t)x[i] << (8 * (j - 4));
            }
        }
        const uint32_t ql = ((lo >> 4) & 0x08080808u) | (lo & 0x07070707u);
        const uint32_t qh = ((hi >> 4) & 0x08080808u) | (hi & 0x07070707u);
        plane[g] = ql | (qh << 4);
    }
}

} // namespace

extern "C" {

int ecf8_encode_bound(uint64_t rows, uint64_t cols, const ecf8_encode_opts *opts, uint64_t *bytes)
{
    if (!bytes) return ECF8_E_ARG;
    return ecf8_internal::encode_bound(rows, cols, opts, bytes);
}

int ecf8_encode_gpu(const void *d_fp8, uint64_t rows, uint64_t cols, const ecf8_encode_opts *opts, void *d_blob,
                    uint64_t blob_capacity, ecf8_header *hdr_out, void *stream)
{
    if (!d_fp8 || !d_blob || !hdr_out) return ECF8_E_ARG;
    uint32_t N, group, lmax, tile_rows, tmode;
    int rc = ecf8_internal::check_options(rows, cols, opts, &N, &group, &lmax, &tile_rows, &tmode);
    if (rc) return rc;
    if (((uintptr_t)d_fp8 & 15) || ((uintptr_t)d_blob & 255)) return ECF8_E_ALIGN;
    if (blob_capacity < 256) return ECF8_E_CAPACITY;
    const uint64_t n = rows * cols;
    hipStream_t s = (hipStream_t)stream;
    const uint64_t blob = (uint64_t)(uintptr_t)d_blob, x = (uint64_t)(uintptr_t)d_fp8;

    // pass 1: histogram, counted into the header's freq[] field
    hipLaunchKernelGGL(fill_zero_kernel, dim3(1), dim3(256), 0, s, blob, (uint64_t)256);
    int g = grid_for_bytes(n / 16 + 1, 256);
    if (g <= 0) return ECF8_E_HIP;
    hipLaunchKernelGGL(histogram_kernel, dim3(g), dim3(256), 0, s, x, n, blob + 128);
    uint64_t freq[16];
    if (hipMemcpyAsync(freq, (const uint8_t *)d_blob + 128, sizeof(freq), hipMemcpyDeviceToHost, s) != hipSuccess)
        return ECF8_E_HIP;
    if (hipStreamSynchronize(s) != hipSuccess) return ECF8_E_HIP;

    ecf8_internal::Plan plan;
    rc = ecf8_internal::plan_encode(freq, rows, cols, opts, &plan);
    if (rc) return rc;
    const ecf8_header &h = plan.hdr;
    if (h.total_size > blob_capacity) return ECF8_E_CAPACITY;

    EncArgs a{};
    a.x = x;
    a.blob = blob;
    a.n = n;
    a.cols = cols;
    a.n_chunks = h.n_chunks;
    a.off_cb = h.off_chunk_bit;
    a.off_lb = h.off_lane_bits;
    a.off_st = h.off_stream;
    a.off_pl = h.off_plane;
    a.st_bytes = h.stream_bytes;
    a.N = N;
    a.group = group;
    a.tiled = tile_rows ? 1 : 0;
    for (int i = 0; i < 16; i++) {
        a.len_packed |= (uint64_t)h.code_len[i] << (4 * i);
        a.code[i] = plan.code[i];
        a.rcode[i] = plan.rcode[i];
    }
    // pass 2: the container
    g = grid_for_bytes(h.total_size / 16, 256);
    hipLaunchKernelGGL(fill_zero_kernel, dim3(g), dim3(256), 0, s, blob, h.total_size);
    hipLaunchKernelGGL(header_kernel, dim3(1), dim3(1024), 0, s, blob, h);
    const uint32_t chunk_blocks = (uint32_t)((h.n_chunks + 3) / 4);
    hipLaunchKernelGGL(lane_bits_kernel, dim3(chunk_blocks), dim3(256), 0, s, a);
    hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(1024), 0, s, blob + h.off_chunk_bit, h.n_chunks);
    // span of a chunk: at most 64 N lmax bits plus the bits before it in its first dword
    const uint32_t need_dw = (64u * N * lmax + 31) / 32 + 2;
    if (need_dw <= 1024) hipLaunchKernelGGL(pack_kernel<1024>, dim3(chunk_blocks), dim3(256), 0, s, a);
    else if (need_dw <= 2048) hipLaunchKernelGGL(pack_kernel<2048>, dim3(chunk_blocks), dim3(256), 0, s, a);
    else hipLaunchKernelGGL(pack_kernel<3848>, dim3(chunk_blocks), dim3(256), 0, s, a);
    g = grid_for_bytes((n + 7) / 8, 256);
    hipLaunchKernelGGL(plane_kernel, dim3(g), dim3(256), 0, s, a);
    if (hipGetLastError() != hipSuccess) return ECF8_E_HIP;
    *hdr_out = h;
    return ECF8_OK;
}

} // extern "C"
