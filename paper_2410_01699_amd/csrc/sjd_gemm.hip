// Skinny-M linear layers of the window forward (paper Sec. 4.1 Step 2): C[M x N] = A[M x K] * W^T
// with M = window size (<= 32).  At this shape every projection is a weight stream: each weight
// element is read from HBM once and used for M multiply-adds, so the kernel is built around
// keeping enough 16-byte loads in flight, not around MFMA throughput.
//
// bf16: W is pre-packed into 16x32 MFMA tiles (see SjdLinear) so that one wave-wide 16-byte-per-lane
// load fetches 1 KiB of contiguous HBM and lands directly in the A-operand registers of
// v_mfma_f32_16x16x32_bf16; the activations are the B operand (tokens along the 16 columns), read
// from L2 as two bf16 planes (hi + lo, see the element-wise kernels) and multiplied separately.  Each wave owns `TN` output tiles and one k-slice; slices write separate fp32 partial
// sums that the consuming element-wise kernel adds in a fixed order (deterministic, no atomics).
// fp32: plain FMA dot products, one output feature per wave (used by the small fp32 models only).
#include "sjd_internal.h"

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

template <int MT, int TN>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(const bf16_t *__restrict__ Wp, const bf16_t *__restrict__ A,
                                                        int N, int K, int kt_per_slice, int n_slices,
                                                        float *__restrict__ part, const SjdState *st)
{
    if (st && st->done) return;
    const int lane = threadIdx.x & 63;
    const int wave_global = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int n_groups = N / (16 * TN);
    const int group = wave_global % n_groups;
    const int slice = wave_global / n_groups;
    if (slice >= n_slices) return;
    const int KT = K / 32;
    const int kt0 = slice * kt_per_slice;
    const int kt1 = min(KT, kt0 + kt_per_slice);

    f32x4 acc[MT][TN];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) acc[mt][tn] = (f32x4){0.f, 0.f, 0.f, 0.f};

    // lane l: weight row l%16 of the tile / token l%16, k-offset (l/16)*8 within the 32-chunk
    const bf16x8 *wbase[TN];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
        wbase[tn] = reinterpret_cast<const bf16x8 *>(Wp) + ((size_t)(group * TN + tn) * KT) * 64 + lane;
    const bf16_t *abase = A + (size_t)(lane & 15) * K + (lane >> 4) * 8;
    const size_t plane = (size_t)SJD_ROWS_MAX * K;    // activations: hi plane, then lo plane

#pragma unroll 4
    for (int kt = kt0; kt < kt1; ++kt) {
        bf16x8 b[MT], bl[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            b[mt] = *reinterpret_cast<const bf16x8 *>(abase + (size_t)mt * 16 * K + (size_t)kt * 32);
            bl[mt] = *reinterpret_cast<const bf16x8 *>(abase + plane + (size_t)mt * 16 * K + (size_t)kt * 32);
        }
        bf16x8 a[TN];
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) a[tn] = __builtin_nontemporal_load(wbase[tn] + (size_t)kt * 64);
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
            {
                acc[mt][tn] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[tn], b[mt], acc[mt][tn], 0, 0, 0);
                acc[mt][tn] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[tn], bl[mt], acc[mt][tn], 0, 0, 0);
            }
    }

    // D[i][j]: lane holds i = (l/16)*4 + 0..3 (output feature within the tile), j = l%16 (token)
    float *out = part + (size_t)slice * (MT * 16) * N;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            float *dst = out + (size_t)(mt * 16 + (lane & 15)) * N + (group * TN + tn) * 16 + (lane >> 4) * 4;
            *reinterpret_cast<f32x4 *>(dst) = acc[mt][tn];
        }
}

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

// row-major [N][K] bf16 -> MFMA streaming order
__global__ void repack_bf16_kernel(const bf16_t *__restrict__ src, bf16_t *__restrict__ dst, int N, int K)
{
    const int KT = K / 32;
    const size_t total = (size_t)N * K / 8;   // 16-byte groups
    for (size_t g = (size_t)blockIdx.x * blockDim.x + threadIdx.x; g < total; g += (size_t)gridDim.x * blockDim.x) {
        const int l = (int)(g & 63);
        const size_t tile = g >> 6;
        const int kt = (int)(tile % KT);
        const size_t nt = tile / KT;
        const bf16_t *s = src + (nt * 16 + (l & 15)) * (size_t)K + (size_t)kt * 32 + (l >> 4) * 8;
        reinterpret_cast<uint4 *>(dst)[g] = *reinterpret_cast<const uint4 *>(s);
    }
}

int sjd_repack_bf16(const bf16_t *src_dev, bf16_t *dst_dev, int32_t N, int32_t K, hipStream_t s)
{
    if (N % 16 || K % 32) return SJD_EINVAL;
    hipLaunchKernelGGL(repack_bf16_kernel, dim3(2048), dim3(256), 0, s, src_dev, dst_dev, N, K);
    HIP_TRY(hipGetLastError());
    return SJD_OK;
}

// Pick tiles-per-wave and the number of k-slices so that about 8 waves per CU stream weights.
void sjd_choose_split(SjdLinear *lin)
{
    const int target_waves = 256 * 8;
    const int nt = lin->N / 16, KT = lin->K / 32;
    lin->tn = (nt % 2 == 0 && nt >= 512) ? 2 : 1;
    const int groups = nt / lin->tn;
    int s = (target_waves + groups - 1) / groups;
    if (s < 1) s = 1;
    int max_s = KT / 8;            // keep at least 8 k-steps (8 KiB per tile stream) per wave
    if (max_s < 1) max_s = 1;
    if (s > max_s) s = max_s;
    if (s > 16) s = 16;
    const int per = (KT + s - 1) / s;
    lin->split_k = (KT + per - 1) / per;
}

size_t sjd_part_stride(const SjdLinear *lin, int32_t rows) { return (size_t)(rows <= 16 ? 16 : 32) * lin->N; }

int sjd_launch_gemm(int32_t dtype, const SjdLinear *lin, const void *act, int32_t rows, float *part,
                    const SjdState *st, hipStream_t s)
{
    if (rows < 1 || rows > SJD_ROWS_MAX) return SJD_EINVAL;
    const int N = lin->N, K = lin->K;
    if (dtype == 0) {
        if (K % 4) return SJD_EINVAL;
        dim3 grid((N + 3) / 4), block(256);
        const float *W = (const float *)lin->w, *A = (const float *)act;
        if (rows <= 8) hipLaunchKernelGGL(gemm_f32_kernel<8>, grid, block, 0, s, W, A, N, K, part, st);
        else if (rows <= 16) hipLaunchKernelGGL(gemm_f32_kernel<16>, grid, block, 0, s, W, A, N, K, part, st);
        else hipLaunchKernelGGL(gemm_f32_kernel<32>, grid, block, 0, s, W, A, N, K, part, st);
        HIP_TRY(hipGetLastError());
        return SJD_OK;
    }
    if (N % (16 * lin->tn) || K % 32) return SJD_EINVAL;
    const int KT = K / 32;
    const int per = (KT + lin->split_k - 1) / lin->split_k;
    const int groups = N / (16 * lin->tn);
    const int waves = groups * lin->split_k;
    dim3 grid((waves + 3) / 4), block(256);
    const bf16_t *W = (const bf16_t *)lin->w, *A = (const bf16_t *)act;
#define GO(MT, TN) hipLaunchKernelGGL((gemm_bf16_kernel<MT, TN>), grid, block, 0, s, W, A, N, K, per, lin->split_k, part, st)
    if (rows <= 16) { if (lin->tn == 2) GO(1, 2); else GO(1, 1); }
    else { if (lin->tn == 2) GO(2, 2); else GO(2, 1); }
#undef GO
    HIP_TRY(hipGetLastError());
    return SJD_OK;
}
