// Fused ECF8 decode + FP8 GEMM for small batches on gfx950 (MI355X), and the
// same GEMM on uncompressed FP8 weights for comparison.
//
//   Y[m][n] = sum_k X[m][k] * W[n][k],   X: M x K FP8 E4M3 (M <= 64),
//   W: rows x K FP8 E4M3 (the compressed tensor), Y: M x rows fp32.
//
// The paper materialises a layer's weights in a buffer and lets the framework's
// GEMM read them back (Section 3.3).  At small M that GEMM is bound by reading
// W, so here the decoded weights never leave the registers they are decoded
// into.  The blob is in the row-tiled layout: a chunk is a block of 16 rows x
// 256 columns of W (64 symbols per lane), lane l decodes row l % 16, and the 16
// bytes it finishes every four steps are columns 64 q + 16 (l / 16) .. + 16 of
// the block.  Eight consecutive K-elements of row l % 16 in lane l is exactly
// a lane's share of the B operand of v_mfma_f32_16x16x32_fp8_fp8 (the order of
// the k's inside an MFMA step is free as long as A and B agree), so a decoded
// piece goes from the merge straight into two MFMAs; X is the A operand, the
// wave's K slice of it held in registers for the whole kernel.  No tile in LDS,
// no barrier between decode and multiply.  This is the only place the matrix
// cores are used.
//
// A workgroup walks over blocks of 16 rows; its NW waves split K (16 chunks per
// block at K = 4096), each wave prefetches its next chunk's payload one chunk
// ahead and the metadata two ahead.  Per block the waves' partial sums meet in
// LDS (double buffered, one barrier per block) and 16 x M outputs are written.
// The kernels need capped codes (no codeword over TB/2 bits: every pair is one
// table hit, and a chunk's span always fits its stage), so they have no second
// level and no fallback path.
//
// In this file: the K = 4096 kernels (X resident in registers) and their twins on
// uncompressed W; the any-K kernels (X fetched chunk by chunk; at short K the waves
// form groups with a block of rows each); scales per 128 x 128 block of W and per
// row or 1 x 128 group of X (ChunkSums); split K for matrices of few rows
// (reduce_split: partial sums and arrival counters in a caller-provided workspace);
// a group of matrices in one launch (ecf8_gemm_grouped_kernel); the host side of
// all of them.
#include "ecf8_gemm_kernels.h"

namespace {

// Split K without a caller workspace (ecf8_gemm_fp8_splitk_static): the arrival counters and partial sums
// live in this array, one copy per GPU, held until the process ends.  Size: the counters plus the largest
// workspace any shape can ask for on a device of up to 256 compute units (blocks x slices <= compute
// units, four tiles of 16 x 16 fp32 at M = 64).  Zero when the module is loaded, and every completed call
// leaves the counters at zero.
constexpr uint64_t STATIC_WS_BYTES = CTR_BYTES + 256ull * 4 * 1024;
static __device__ __align__(256) uint8_t scratch[STATIC_WS_BYTES];

// Device address of `scratch` on the current device (the array's name is only a host-side handle), looked
// up once per device; *first tells the caller that this device's copy has not been used yet.
void *static_scratch(bool *first)
{
    static std::mutex m;
    static void *ptr[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
    std::lock_guard<std::mutex> lk(m);
    *first = false;
    if (!ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
        ptr[dev] = p;
        *first = true;
    }
    return ptr[dev];
}

} // namespace

extern "C" {

int ecf8_gemm_fp8(const ecf8_header *h, const void *d_blob, const void *d_x, uint32_t M, float *d_y, void *stream)
{
    GArgs a;
    int rc = fused_args(h, d_blob, d_x, M, d_y, &a);
    return rc ? rc : launch_fused<0>(a, stream);
}

int ecf8_gemm_fp8_raw(const void *d_w, uint64_t rows, uint64_t cols, const void *d_x, uint32_t M, float *d_y,
                      void *stream)
{
    GArgs a;
    int rc = raw_args(d_w, rows, cols, d_x, M, d_y, &a);
    return rc ? rc : launch_raw<0>(a, stream);
}

int ecf8_gemm_fp8_scaled(const ecf8_header *h, const void *d_blob, const void *d_x, uint32_t M, const float *d_w_scale,
                         const float *d_x_scale, uint32_t x_scale_cols, float *d_y, void *stream)
{
    GArgs a;
    int rc = fused_args(h, d_blob, d_x, M, d_y, &a);
    if (!rc) rc = scale_args(d_w_scale, d_x_scale, x_scale_cols, &a);
    if (rc) return rc;
    return a.xs_cols > 1 ? launch_fused<2>(a, stream) : launch_fused<1>(a, stream);
}

int ecf8_gemm_fp8_raw_scaled(const void *d_w, uint64_t rows, uint64_t cols, const void *d_x, uint32_t M,
                             const float *d_w_scale, const float *d_x_scale, uint32_t x_scale_cols, float *d_y, void *stream)
{
    GArgs a;
    int rc = raw_args(d_w, rows, cols, d_x, M, d_y, &a);
    if (!rc) rc = scale_args(d_w_scale, d_x_scale, x_scale_cols, &a);
    if (rc) return rc;
    return a.xs_cols > 1 ? launch_raw<2>(a, stream) : launch_raw<1>(a, stream);
}

int ecf8_gemm_splitk_plan(uint64_t rows, uint64_t cols, uint32_t M, uint32_t compute_units, uint32_t *slices,
                          uint64_t *workspace_bytes_out)
{
    if (cols == 0 || cols % 256 || cols > (1u << 20) || rows == 0 || rows % BLOCK_ROWS || M == 0 || M > 64) return ECF8_E_ARG;
    int cus = (int)compute_units;
    if (cus == 0) cus = device_cus();
    if (cus <= 0) return ECF8_E_HIP;
    const uint32_t sl = pick_slices(rows, cols, cus);
    if (slices) *slices = sl;
    if (workspace_bytes_out) *workspace_bytes_out = workspace_bytes(rows, M, sl);
    return ECF8_OK;
}

uint32_t ecf8_gemm_splitk_slices(uint64_t rows, uint64_t cols)
{
    uint32_t sl = 0;
    return ecf8_gemm_splitk_plan(rows, cols, 1, 0, &sl, nullptr) == ECF8_OK ? sl : 0;
}

uint64_t ecf8_gemm_splitk_workspace_bytes(uint64_t rows, uint64_t cols, uint32_t M)
{
    uint64_t bytes = 0;
    return ecf8_gemm_splitk_plan(rows, cols, M, 0, nullptr, &bytes) == ECF8_OK ? bytes : 0;
}

int ecf8_gemm_splitk_workspace_init(void *d_workspace, uint64_t bytes, void *stream)
{
    if (bytes == 0) return ECF8_OK;
    if (!d_workspace) return ECF8_E_ARG;
    if (((uintptr_t)d_workspace & 15) || (bytes & 3)) return ECF8_E_ALIGN;
    const uint64_t n = bytes / 4;
    if ((n + 255) / 256 > 0x7fffffffull) return ECF8_E_ARG;
    hipLaunchKernelGGL(gemm_fill_zero_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                       (uint64_t)(uintptr_t)d_workspace, n);
    return hipGetLastError() == hipSuccess ? ECF8_OK : ECF8_E_HIP;
}

int ecf8_gemm_fp8_splitk(const ecf8_header *h, const void *d_blob, const void *d_x, uint32_t M, const float *d_w_scale,
                         const float *d_x_scale, uint32_t x_scale_cols, float *d_y, void *d_workspace,
                         uint64_t workspace_bytes_, void *stream)
{
    GArgs a;
    const int rc = fused_args(h, d_blob, d_x, M, d_y, &a);
    return rc ? rc : run_split<false>(a, d_w_scale, d_x_scale, x_scale_cols, d_workspace, workspace_bytes_, stream);
}

int ecf8_gemm_fp8_splitk_static(const ecf8_header *h, const void *d_blob, const void *d_x, uint32_t M, const float *d_w_scale,
                                const float *d_x_scale, uint32_t x_scale_cols, float *d_y, void *stream)
{
    GArgs a;
    const int rc = fused_args(h, d_blob, d_x, M, d_y, &a);
    if (rc) return rc;
    const int cus = device_cus();
    if (cus <= 0) return ECF8_E_HIP;
    if (workspace_bytes(a.rows, M, pick_slices(a.rows, a.K, cus)) > STATIC_WS_BYTES) return ECF8_E_CAPACITY;
    bool first = false;
    void *ws = static_scratch(&first);
    if (!ws) return ECF8_E_HIP;
    if (first) {      // counters start at zero (a fill kernel, not a memset: the call may be under graph capture)
        hipLaunchKernelGGL(gemm_fill_zero_kernel, dim3((unsigned)(CTR_BYTES / 4 / 256)), dim3(256), 0, (hipStream_t)stream,
                           (uint64_t)(uintptr_t)ws, CTR_BYTES / 4);
        if (hipGetLastError() != hipSuccess) return ECF8_E_HIP;
    }
    return run_split<false>(a, d_w_scale, d_x_scale, x_scale_cols, ws, STATIC_WS_BYTES, stream);
}

int ecf8_gemm_fp8_raw_splitk(const void *d_w, uint64_t rows, uint64_t cols, const void *d_x, uint32_t M,
                             const float *d_w_scale, const float *d_x_scale, uint32_t x_scale_cols, float *d_y,
                             void *d_workspace, uint64_t workspace_bytes_, void *stream)
{
    GArgs a;
    const int rc = raw_args(d_w, rows, cols, d_x, M, d_y, &a);
    return rc ? rc : run_split<true>(a, d_w_scale, d_x_scale, x_scale_cols, d_workspace, workspace_bytes_, stream);
}

int ecf8_gemm_group_prepare(const ecf8_gemm_group_desc *descs, uint32_t n, ecf8_gemm_group_item *items_host,
                            ecf8_gemm_group_info *info)
{
    if (!descs || !items_host || !info || n == 0) return ECF8_E_ARG;
    std::memset(info, 0, sizeof(*info));
    std::memset(items_host, 0, sizeof(*items_host) * n);
    const bool raw = descs[0].hdr == nullptr;
    uint32_t mode = 0, max_M = 0;
    uint64_t work = 0;
    for (uint32_t i = 0; i < n; i++) {
        const ecf8_gemm_group_desc &d = descs[i];
        if ((d.hdr == nullptr) != raw) return ECF8_E_ARG;           // all compressed, or all uncompressed
        GItem it{};
        int rc = raw ? raw_args(d.d_w, d.rows, d.cols, d.d_x, d.M, d.d_y, &it.a) : fused_args(d.hdr, d.d_w, d.d_x, d.M, d.d_y, &it.a);
        if (rc) return rc;
        uint32_t m = 0;
        if (d.d_w_scale || d.d_x_scale || d.x_scale_cols) {
            rc = scale_args(d.d_w_scale, d.d_x_scale, d.x_scale_cols, &it.a);
            if (rc) return rc;
            m = it.a.xs_cols > 1 ? 2 : 1;
        }
        if (i == 0) mode = m;
        else if (m != mode) return ECF8_E_ARG;                      // one kind of scales per group
        it.first_work = work;
        work += it.a.rows / BLOCK_ROWS * (it.a.K / 256);
        if (d.M > max_M) max_M = d.M;
        std::memcpy(&items_host[i], &it, sizeof(it));
    }
    info->total_work = work;
    info->n_items = n;
    info->max_M = max_M;
    info->scale_mode = mode;
    info->raw = raw ? 1u : 0u;
    return ECF8_OK;
}

int ecf8_gemm_fp8_grouped(const ecf8_gemm_group_item *d_items, const ecf8_gemm_group_info *info, void *stream)
{
    if (!d_items || !info || info->n_items == 0 || info->total_work == 0 || info->max_M == 0 || info->max_M > 64 ||
        info->scale_mode > 2 || info->raw > 1)
        return ECF8_E_ARG;
    if ((uintptr_t)d_items & 7) return ECF8_E_ALIGN;
    GGArgs g{(uint64_t)(uintptr_t)d_items, info->n_items, info->total_work};
    const uint32_t M = info->max_M;
    if (info->raw)
        return info->scale_mode == 0 ? launch_grouped<0, true>(g, M, stream)
             : info->scale_mode == 1 ? launch_grouped<1, true>(g, M, stream) : launch_grouped<2, true>(g, M, stream);
    return info->scale_mode == 0 ? launch_grouped<0, false>(g, M, stream)
         : info->scale_mode == 1 ? launch_grouped<1, false>(g, M, stream) : launch_grouped<2, false>(g, M, stream);
}

} // extern "C"
