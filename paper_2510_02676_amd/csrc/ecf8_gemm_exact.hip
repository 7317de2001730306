// The fused ECF8 decode + GEMM calls that multiply on the F16 matrix cores (ACC = 1 of the kernels in
// ecf8_gemm_kernels.h): decoded E4M3 bytes and the E4M3 bytes of X are converted to halves in registers,
// which is exact, so every product is exact and the sums are plain fp32 sums.  Same decode, same
// workgroup shapes, same order of accumulation as the FP8 matrix-core calls in ecf8_gemm.hip; the twin
// on uncompressed weights agrees with the fused call bit for bit here too.
#include "ecf8_gemm_kernels.h"

namespace {

template <bool RAW>
int run_exact(GArgs &a, const float *d_w_scale, const float *d_x_scale, uint32_t x_scale_cols, void *stream)
{
    int sc = 0;
    if (d_w_scale || d_x_scale || x_scale_cols) {
        const int rc = scale_args(d_w_scale, d_x_scale, x_scale_cols, &a);
        if (rc) return rc;
        sc = a.xs_cols > 1 ? 2 : 1;
    }
    if constexpr (RAW) return sc == 0 ? launch_raw<0, 1>(a, stream) : sc == 1 ? launch_raw<1, 1>(a, stream) : launch_raw<2, 1>(a, stream);
    else return sc == 0 ? launch_fused<0, 1>(a, stream) : sc == 1 ? launch_fused<1, 1>(a, stream) : launch_fused<2, 1>(a, stream);
}

} // namespace

extern "C" {

int ecf8_gemm_fp8_exact(const ecf8_header *h, const void *d_blob, const void *d_x, uint32_t M, const float *d_w_scale,
                        const float *d_x_scale, uint32_t x_scale_cols, float *d_y, void *stream)
{
    GArgs a;
    const int rc = fused_args(h, d_blob, d_x, M, d_y, &a);
    return rc ? rc : run_exact<false>(a, d_w_scale, d_x_scale, x_scale_cols, stream);
}

int ecf8_gemm_fp8_raw_exact(const void *d_w, uint64_t rows, uint64_t cols, const void *d_x, uint32_t M,
                            const float *d_w_scale, const float *d_x_scale, uint32_t x_scale_cols, float *d_y, void *stream)
{
    GArgs a;
    const int rc = raw_args(d_w, rows, cols, d_x, M, d_y, &a);
    return rc ? rc : run_exact<true>(a, d_w_scale, d_x_scale, x_scale_cols, stream);
}

} // extern "C"
