// fp32 linear layers of the window forward (paper Sec. 4.1 Step 2) for the small fp32 models:
// C[M x N] = A[M x K] * W^T with plain FMA dot products, one output feature per wave.  These models
// are launch-bound; the bf16 weight-streaming kernel lives in sjd_gemm_bf16.hip.
#include "sjd_internal.h"

// fp32: out[m][n] = sum_k A[m][k] W[n][k]; one wave per output feature, lanes split k by float4
template <int MR>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float *__restrict__ W, const float *__restrict__ A, int N,
                                                       int K, float *__restrict__ out, const SjdState *st)
{
    if (st && st->done) return;
    const int lane = threadIdx.x & 63;
    const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (n >= N) return;
    float acc[MR];
#pragma unroll
    for (int m = 0; m < MR; ++m) acc[m] = 0.f;
    const float4 *w4 = reinterpret_cast<const float4 *>(W + (size_t)n * K);
    for (int k4 = lane; k4 < K / 4; k4 += 64) {
        const float4 w = w4[k4];
#pragma unroll
        for (int m = 0; m < MR; ++m) {
            const float4 a = reinterpret_cast<const float4 *>(A + (size_t)m * K)[k4];
            acc[m] = fmaf(w.x, a.x, fmaf(w.y, a.y, fmaf(w.z, a.z, fmaf(w.w, a.w, acc[m]))));
        }
    }
#pragma unroll
    for (int m = 0; m < MR; ++m) {
        float v = acc[m];
        for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
        if (lane == 0) out[(size_t)m * N + n] = v;
    }
}

int sjd_launch_gemm(int32_t dtype, const SjdLinear *lin, const void *act, int32_t rows, float *part,
                    const SjdState *st, hipStream_t s)
{
    if (rows < 1 || rows > SJD_ROWS_F32) return SJD_EINVAL;
    const int N = lin->N, K = lin->K;
    if (dtype == 0) {
        if (K % 4) return SJD_EINVAL;
        dim3 grid((N + 3) / 4), block(256);
        const float *W = (const float *)lin->w, *A = (const float *)act;
        if (rows <= 8) SJD_LAUNCH(gemm_f32_kernel<8>, grid, block, 0, s, W, A, N, K, part, st);
        else if (rows <= 16) SJD_LAUNCH(gemm_f32_kernel<16>, grid, block, 0, s, W, A, N, K, part, st);
        else SJD_LAUNCH(gemm_f32_kernel<32>, grid, block, 0, s, W, A, N, K, part, st);
        HIP_TRY(hipGetLastError());
        return SJD_OK;
    }
    return SJD_EINVAL;   // bf16 models use sjd_launch_gemm_bf16
}
