// GPU-side encoder of the wide-alphabet codec (E5M2, BF16) for gfx950: Section 3.1 on the device
// for 5- and 8-bit exponent fields.  Writes exactly the container ecfw_encode writes, byte for byte:
// the code and the layout come from the same host routine, fed with the device histogram.
//
//   histogram (LDS counters, a few copies to spread the hot bins; one atomic add per bin per
//   workgroup into the blob's own freq section) -> [host: the histogram back, code + layout]
//   -> fill 0 (everything but freq), header + code lengths -> lane_bits and chunk totals (one wave
//   per chunk) -> prefix sum of the totals -> stream (one wave per chunk assembles its span in LDS
//   with ds_or and copies it out; the two dwords a span may share with its neighbours go out with
//   atomic OR) -> planes of the remaining bits.
// No scratch memory: the histogram is counted into the freq section and the chunk totals into
// chunk_bit[], both part of the output.
#include "ecfw.h"

#include "ecf8_enc_device.h"
#include "ecfw_plan.h"

namespace {

struct WEncArgs {
    uint64_t x, blob;                     // device addresses
    uint64_t n, n_chunks;
    uint64_t off_len, off_cb, off_lb, off_st, off_pl, off_sg;
    uint32_t N, group;
};

template <int FMT> struct EFmt;
template <> struct EFmt<ECFW_FMT_E5M2> { static constexpr int P = 16, ELEM = 1, A = 32; };
template <> struct EFmt<ECFW_FMT_BF16> { static constexpr int P = 8, ELEM = 2, A = 256; };

// exponent field of element i
template <int FMT>
__device__ __forceinline__ uint32_t sym_of(const GLOBAL uint8_t *x, uint64_t i)
{
    if (FMT == ECFW_FMT_E5M2) return (x[i] >> 2) & 31u;
    return (((const GLOBAL uint16_t *)x)[i] >> 7) & 255u;
}

// element index of piece q of lane l of chunk c (see the stream section of ecfw.h)
template <int FMT>
__device__ __forceinline__ uint64_t piece_start(const WEncArgs &a, uint64_t c, uint32_t l, uint32_t q)
{
    constexpr uint64_t P = EFmt<FMT>::P;
    const uint64_t E = 64ull * a.N;
    const uint64_t grouped = (a.n / E) & ~((uint64_t)a.group - 1);
    if (c < grouped) {
        const uint64_t w = c & (a.group - 1);
        return (c - w) * E + w * 64 * P + (uint64_t)q * a.group * 64 * P + l * P;
    }
    return c * E + q * 64 * P + l * P;
}

// Histogram of the exponent field into A u64 counters.  COPIES histograms per workgroup in LDS
// (lane % COPIES picks one) keep the lanes of a wave off each other when most elements share a
// handful of exponents; one atomic add per bin per workgroup at the end.
template <int FMT>
__global__ __launch_bounds__(256) void w_histogram_kernel(uint64_t x_, uint64_t n, uint64_t counters_)
{
    constexpr int A = EFmt<FMT>::A, COPIES = 16;
    __shared__ uint32_t cnt[A * COPIES];
    const GLOBAL uint8_t *x = (const GLOBAL uint8_t *)x_;
    GLOBAL unsigned long long *counters = (GLOBAL unsigned long long *)counters_;
    const int tid = threadIdx.x, copy = tid & (COPIES - 1);
    for (int i = tid; i < A * COPIES; i += 256) cnt[i] = 0;
    __syncthreads();
    // 16 bytes per thread and step: 16 E5M2 or 8 BF16 elements
    constexpr uint64_t PER = 16 / EFmt<FMT>::ELEM;
    const uint64_t n16 = n / PER;
    for (uint64_t i = (uint64_t)blockIdx.x * 256 + tid; i < n16; i += (uint64_t)gridDim.x * 256) {
        const u32x4 v = __builtin_nontemporal_load((const GLOBAL u32x4 *)x + i);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int k = 0; k < 4; k++) {
            if (FMT == ECFW_FMT_E5M2) {
#pragma unroll
                for (int b = 0; b < 4; b++) atomicAdd(&cnt[((w[k] >> (8 * b + 2)) & 31u) * COPIES + copy], 1u);
            } else {
                atomicAdd(&cnt[((w[k] >> 7) & 255u) * COPIES + copy], 1u);
                atomicAdd(&cnt[((w[k] >> 23) & 255u) * COPIES + copy], 1u);
            }
        }
    }
    if (blockIdx.x == 0)
        for (uint64_t i = n16 * PER + tid; i < n; i += 256) atomicAdd(&cnt[sym_of<FMT>(x, i) * COPIES + copy], 1u);
    __syncthreads();
    for (int s = tid; s < A; s += 256) {
        unsigned long long sum = 0;
        for (int k = 0; k < COPIES; k++) sum += cnt[s * COPIES + k];
        if (sum) atomicAdd((unsigned long long *)(counters + s), sum);
    }
}

struct WHeadArgs {
    ecfw_header h;
    uint8_t len[256];
};

// Header and code lengths (the freq section already holds the histogram).
__global__ __launch_bounds__(128) void w_header_kernel(uint64_t blob_, WHeadArgs a)
{
    GLOBAL uint32_t *blob = (GLOBAL uint32_t *)blob_;
    const int tid = threadIdx.x;
    if (tid < 64) blob[tid] = ((const uint32_t *)&a.h)[tid];
    if ((uint32_t)tid * 4 < a.h.n_alphabet) blob[a.h.off_code_len / 4 + tid] = ((const uint32_t *)a.len)[tid];
}

// lane_bits[c][l] = code bits of the lane's symbols; chunk_bit[c + 1] = bits of chunk c (turned into
// stream positions by the scan).  One wave per chunk.
template <int FMT>
__global__ __launch_bounds__(256) void w_lane_bits_kernel(WEncArgs a)
{
    constexpr int P = EFmt<FMT>::P, A = EFmt<FMT>::A;
    __shared__ uint8_t s_len[256];
    for (int i = threadIdx.x; i < 256; i += 256) s_len[i] = i < A ? ((const GLOBAL uint8_t *)(a.blob + a.off_len))[i] : 0;
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const uint64_t c = (uint64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (c >= a.n_chunks) return;
    const GLOBAL uint8_t *x = (const GLOBAL uint8_t *)a.x;
    uint32_t lb = 0;
    for (uint32_t q = 0; q < a.N / P; q++) {
        const uint64_t e = piece_start<FMT>(a, c, lane, q);
        for (uint32_t j = 0; j < (uint32_t)P && e + j < a.n; j++) lb += s_len[sym_of<FMT>(x, e + j)];
    }
    ((GLOBAL uint16_t *)(a.blob + a.off_lb))[c * 64 + lane] = (uint16_t)lb;
    const uint32_t total = wave_incl_scan(lb);
    if (lane == 63) ((GLOBAL uint64_t *)(a.blob + a.off_cb))[c + 1] = total;
}

// Stream: one wave per chunk.  The workgroup first derives the
// canonical codewords from the code lengths (every thread its own symbol: all shorter codes come
// before it, and the codes of its length with a smaller symbol), then walks over its chunks: the
// span's dwords are assembled in LDS (every lane ORs its codewords in: forward run up from its
// first bit, backward run down from its last) and copied out; the first and the last dword of a
// span can hold bits of neighbouring chunks and go out with atomic OR onto the zeroed stream.
template <int FMT, int STAGE_DWORDS, int WPB>      // WPB waves per workgroup: as many stages as fit 64 KiB of LDS
__global__ __launch_bounds__(WPB * 64) void w_pack_kernel(WEncArgs a)
{
    constexpr int P = EFmt<FMT>::P, A = EFmt<FMT>::A;
    __shared__ uint32_t stage_all[WPB][STAGE_DWORDS];
    __shared__ uint8_t s_len[256];
    __shared__ uint32_t s_code[256], s_rcode[256];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int s = tid; s < 256; s += WPB * 64) s_len[s] = s < A ? ((const GLOBAL uint8_t *)(a.blob + a.off_len))[s] : 0;
    __syncthreads();
    for (int s = tid; s < 256; s += WPB * 64) {
        const uint32_t l = s_len[s];
        uint32_t code = 0;
        if (l) {
            for (int j = 0; j < A; j++) {
                const uint32_t lj = s_len[j];
                if (lj != 0 && lj < l) code += 1u << (l - lj);
                else if (lj == l && j < s) code += 1;
            }
        }
        s_code[s] = code;
        s_rcode[s] = l ? __brev(code) >> (32 - l) : 0;
    }
    __syncthreads();
    uint32_t *stage = stage_all[wave];
    const GLOBAL uint8_t *x = (const GLOBAL uint8_t *)a.x;
    const GLOBAL uint64_t *cb = (const GLOBAL uint64_t *)(a.blob + a.off_cb);
    GLOBAL uint32_t *out = (GLOBAL uint32_t *)(a.blob + a.off_st);
    const uint32_t pieces = a.N / P;
    for (uint64_t c = (uint64_t)blockIdx.x * WPB + wave; c < a.n_chunks; c += (uint64_t)gridDim.x * WPB) {   // wave-uniform
        const uint64_t b0 = cb[c], b1 = cb[c + 1];
        const uint32_t lb = ((const GLOBAL uint16_t *)(a.blob + a.off_lb))[c * 64 + lane];
        const uint64_t first_dw = b0 >> 5, end_dw = (b1 + 31) >> 5;      // dwords [first_dw, end_dw) hold the span
        uint32_t n_dw = (uint32_t)(end_dw - first_dw);
        if (n_dw > (uint32_t)STAGE_DWORDS) n_dw = STAGE_DWORDS;          // cannot happen for a span under the cap
        for (uint32_t i = lane; i < n_dw; i += 64) stage[i] = 0;
        __builtin_amdgcn_wave_barrier();
        uint32_t fwd = (uint32_t)(b0 & 31) + (wave_incl_scan(lb) - lb);  // stage bit of the lane's first bit
        uint32_t bwd = fwd + lb;                                         // one past its last bit
        auto put = [&](uint32_t at, uint32_t bits, uint32_t nb) {
            const uint32_t d = at >> 5, sh = at & 31;
            if (d >= (uint32_t)STAGE_DWORDS) return;
            __hip_atomic_fetch_or(&stage[d], bits << sh, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            if (sh + nb > 32 && d + 1 < (uint32_t)STAGE_DWORDS)
                __hip_atomic_fetch_or(&stage[d + 1], bits >> (32 - sh), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        };
        for (uint32_t q = 0; q < pieces; q++) {
            const uint64_t e = piece_start<FMT>(a, c, lane, q);
            for (uint32_t j = 0; j < (uint32_t)P && e + j < a.n; j++) {
                const uint32_t s = sym_of<FMT>(x, e + j);
                const uint32_t l = s_len[s];
                if (q < pieces / 2) { put(fwd, s_rcode[s], l); fwd += l; }
                else { bwd -= l; put(bwd, s_code[s], l); }
            }
        }
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
        for (uint32_t i = lane; i < n_dw; i += 64) {
            const uint32_t v = stage[i];
            if (i == 0 || i + 1 == n_dw) { if (v) atomicOr((unsigned int *)(out + first_dw + i), v); }
            else out[first_dw + i] = v;
        }
        __builtin_amdgcn_wave_barrier();
    }
}

// BF16 plane: one byte sign << 7 | mantissa per element, the bytes of four elements in the order 0 2 1 3.
__global__ __launch_bounds__(256) void w_plane_bf16_kernel(WEncArgs a)
{
    const GLOBAL uint16_t *x = (const GLOBAL uint16_t *)a.x;
    GLOBAL uint32_t *plane = (GLOBAL uint32_t *)(a.blob + a.off_pl);
    const uint64_t groups = (a.n + 3) / 4;
    for (uint64_t g = (uint64_t)blockIdx.x * 256 + threadIdx.x; g < groups; g += (uint64_t)gridDim.x * 256) {
        uint32_t r[4] = {0, 0, 0, 0};
        for (uint32_t j = 0; j < 4 && g * 4 + j < a.n; j++) {
            const uint32_t v = x[g * 4 + j];
            r[j] = ((v >> 8) & 128u) | (v & 127u);
        }
        plane[g] = r[0] | (r[2] << 8) | (r[1] << 16) | (r[3] << 24);
    }
}

// E5M2 planes: per piece of 16 elements one u32 of mantissas (element 4d + j in bits 8j + 2d) and one
// u16 of signs (bit e = element e).
__global__ __launch_bounds__(256) void w_plane_e5m2_kernel(WEncArgs a)
{
    const GLOBAL uint8_t *x = (const GLOBAL uint8_t *)a.x;
    GLOBAL uint32_t *plane = (GLOBAL uint32_t *)(a.blob + a.off_pl);
    GLOBAL uint16_t *sign = (GLOBAL uint16_t *)(a.blob + a.off_sg);
    const uint64_t pieces = (a.n + 15) / 16;
    for (uint64_t g = (uint64_t)blockIdx.x * 256 + threadIdx.x; g < pieces; g += (uint64_t)gridDim.x * 256) {
        uint32_t m = 0, s = 0;
        for (uint32_t e = 0; e < 16 && g * 16 + e < a.n; e++) {
            const uint32_t b = x[g * 16 + e];
            m |= (b & 3u) << (8 * (e & 3) + 2 * (e >> 2));
            s |= (b >> 7) << e;
        }
        plane[g] = m;
        sign[g] = (uint16_t)s;
    }
}

template <int FMT>
int encode_on_gpu(const void *d_elems, uint64_t rows, uint64_t cols, const ecfw_encode_opts *opts, uint32_t N,
                  uint32_t group, uint32_t lmax, void *d_blob, uint64_t blob_capacity, ecfw_header *hdr_out, hipStream_t s)
{
    constexpr int A = EFmt<FMT>::A;
    const uint64_t n = rows * cols;
    const uint64_t blob = (uint64_t)(uintptr_t)d_blob, x = (uint64_t)(uintptr_t)d_elems;
    // the sections in front of chunk_bit have fixed places: header 256, code_len 256, freq 8A rounded up
    const uint64_t off_freq = 512, fixed = off_freq + (8ull * A + 255) / 256 * 256;
    if (blob_capacity < fixed) return ECF8_E_CAPACITY;

    // pass 1: histogram, counted into the blob's freq section
    hipLaunchKernelGGL(fill_zero_kernel, dim3(1), dim3(256), 0, s, blob, fixed);
    int g = grid_for_bytes(n * EFmt<FMT>::ELEM / 16 + 1, 256);
    if (g <= 0) return ECF8_E_HIP;
    hipLaunchKernelGGL(w_histogram_kernel<FMT>, dim3(g), dim3(256), 0, s, x, n, blob + off_freq);
    uint64_t freq[256] = {};
    if (hipMemcpyAsync(freq, (const uint8_t *)d_blob + off_freq, 8ull * A, hipMemcpyDeviceToHost, s) != hipSuccess)
        return ECF8_E_HIP;
    if (hipStreamSynchronize(s) != hipSuccess) return ECF8_E_HIP;

    ecfw_internal::WPlan plan;
    int rc = ecfw_internal::plan_encode(freq, FMT, rows, cols, N, group, lmax, &plan);
    if (rc) return rc;
    const ecfw_header &h = plan.hdr;
    if (h.total_size > blob_capacity) return ECF8_E_CAPACITY;
    if (h.off_freq != off_freq || h.off_chunk_bit != fixed) return ECF8_E_FORMAT;

    WEncArgs a{};
    a.x = x;
    a.blob = blob;
    a.n = n;
    a.n_chunks = h.n_chunks;
    a.off_len = h.off_code_len;
    a.off_cb = h.off_chunk_bit;
    a.off_lb = h.off_lane_bits;
    a.off_st = h.off_stream;
    a.off_pl = h.off_plane;
    a.off_sg = h.off_sign;
    a.N = N;
    a.group = group;
    // pass 2: the container (everything behind the histogram is zeroed first)
    g = grid_for_bytes((h.total_size - fixed) / 16, 256);
    hipLaunchKernelGGL(fill_zero_kernel, dim3(g), dim3(256), 0, s, blob + fixed, h.total_size - fixed);
    WHeadArgs ha;
    ha.h = h;
    for (int i = 0; i < 256; i++) ha.len[i] = plan.len[i];
    hipLaunchKernelGGL(w_header_kernel, dim3(1), dim3(128), 0, s, blob, ha);
    const uint32_t chunk_blocks = (uint32_t)((h.n_chunks + 3) / 4);
    hipLaunchKernelGGL(w_lane_bits_kernel<FMT>, dim3(chunk_blocks), dim3(256), 0, s, a);
    hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(1024), 0, s, blob + h.off_chunk_bit, h.n_chunks);
    // span of a chunk: at most 64 N lmax bits plus the bits before it in its first dword
    const uint32_t need_dw = (64u * N * h.max_code_len + 31) / 32 + 2;
    const int pg = grid_for_bytes(chunk_blocks, 1);
    if (need_dw <= 1024) hipLaunchKernelGGL((w_pack_kernel<FMT, 1024, 4>), dim3(pg), dim3(256), 0, s, a);
    else if (need_dw <= 2048) hipLaunchKernelGGL((w_pack_kernel<FMT, 2048, 4>), dim3(pg), dim3(256), 0, s, a);
    else hipLaunchKernelGGL((w_pack_kernel<FMT, 4104, 2>), dim3(pg), dim3(128), 0, s, a);
    if (FMT == ECFW_FMT_BF16) {
        g = grid_for_bytes((n + 3) / 4, 256);
        hipLaunchKernelGGL(w_plane_bf16_kernel, dim3(g), dim3(256), 0, s, a);
    } else {
        g = grid_for_bytes((n + 15) / 16, 256);
        hipLaunchKernelGGL(w_plane_e5m2_kernel, dim3(g), dim3(256), 0, s, a);
    }
    if (hipGetLastError() != hipSuccess) return ECF8_E_HIP;
    (void)opts;
    *hdr_out = h;
    return ECF8_OK;
}

} // namespace

extern "C" {

int ecfw_encode_bound(uint64_t rows, uint64_t cols, const ecfw_encode_opts *opts, uint64_t *bytes)
{
    if (!bytes) return ECF8_E_ARG;
    uint32_t N, group, lmax;
    int rc = ecfw_internal::check_options(opts, rows, cols, &N, &group, &lmax);
    if (rc) return rc;
    return ecfw_internal::encode_bound(opts->fmt, rows, cols, N, lmax, bytes);
}

int ecfw_encode_gpu(const void *d_elems, uint64_t rows, uint64_t cols, const ecfw_encode_opts *opts, void *d_blob,
                    uint64_t blob_capacity, ecfw_header *hdr_out, void *stream)
{
    if (!d_elems || !d_blob || !hdr_out) return ECF8_E_ARG;
    uint32_t N, group, lmax;
    int rc = ecfw_internal::check_options(opts, rows, cols, &N, &group, &lmax);
    if (rc) return rc;
    if (((uintptr_t)d_elems & 15) || ((uintptr_t)d_blob & 255)) return ECF8_E_ALIGN;
    hipStream_t s = (hipStream_t)stream;
    return opts->fmt == ECFW_FMT_BF16
               ? encode_on_gpu<ECFW_FMT_BF16>(d_elems, rows, cols, opts, N, group, lmax, d_blob, blob_capacity, hdr_out, s)
               : encode_on_gpu<ECFW_FMT_E5M2>(d_elems, rows, cols, opts, N, group, lmax, d_blob, blob_capacity, hdr_out, s);
}

} // extern "C"
