// Grouped GEMMs of the subnet SGD step (Section 2.1 "Training Subnets"): one
// launch covers all S subnets (group index = blockIdx.z).  Every product of the
// step has the form  C_g[m][n] = sum_k A_g(m,k) * B_g(n,k)  with strided operands:
//   forward        z_l  = h_{l-1} W_l^T      A = h_{l-1} [B][C],  B = W_l [R][C]
//   backward data  dh   = dz_l W_l           A = dz_l [B][R],     B(n,k) = W_l[k][n]
//   backward weight dW  = dz_l^T h_{l-1}     A(m,k) = dz_l[k][m], B(n,k) = h_{l-1}[k][n]
// and a fused epilogue (bias + ReLU, ReLU mask, or the SGD update in place).
//
// This file holds the generic kernel: any strides, any alignment, fp32 FMA with
// LDS tiles.  It is the fallback for shapes the MFMA kernels do not take.
#include <cstdlib>
#include <string>

#include "ist_internal.h"

namespace ist {

constexpr int GBM = 64, GBN = 64, GBK = 16;

template <typename D, int EPI>
__global__ __launch_bounds__(256) void k_gemm_generic(GemmArgs a)
{
    using T = typename D::T;
    __shared__ float As[GBK][GBM + 4];
    __shared__ float Bs[GBK][GBN + 4];
    const int g = blockIdx.z;
    const int m0 = blockIdx.y * GBM, n0 = blockIdx.x * GBN;
    const T *A = static_cast<const T *>(a.A) + (int64_t)g * a.gA;
    const T *B = static_cast<const T *>(a.B) + (int64_t)g * a.gB;
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.0f;

    const bool a_kfast = (a.sak == 1), b_kfast = (a.sbk == 1);
    for (int k0 = 0; k0 < a.K; k0 += GBK) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            int idx = tid + e * 256;
            int mm = a_kfast ? idx / GBK : idx % GBM;
            int kk = a_kfast ? idx % GBK : idx / GBM;
            int m = m0 + mm, k = k0 + kk;
            As[kk][mm] = (m < a.M && k < a.K) ? D::ld(A + (int64_t)m * a.sam + (int64_t)k * a.sak) : 0.0f;
            int nn = b_kfast ? idx / GBK : idx % GBN;
            int kb = b_kfast ? idx % GBK : idx / GBN;
            int n = n0 + nn;
            k = k0 + kb;
            Bs[kb][nn] = (n < a.N && k < a.K) ? D::ld(B + (int64_t)n * a.sbn + (int64_t)k * a.sbk) : 0.0f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < GBK; ++kk) {
            float av[4], bv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) av[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) bv[j] = Bs[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
        }
        __syncthreads();
    }

#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int m = m0 + ty * 4 + i;
        if (m >= a.M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int n = n0 + tx * 4 + j;
            if (n >= a.N) continue;
            float v = EPI == EPI_UPDATE ? acc[i][j] : a.alpha * acc[i][j];
            int64_t ci = (int64_t)g * a.gC + (int64_t)m * a.ldc + n;
            if (EPI == EPI_FWD_RELU) {
                if (a.bias) v += D::ld(static_cast<const T *>(a.bias) + (int64_t)g * a.gBias + n);
                static_cast<T *>(a.C)[ci] = D::cvt(v > 0.0f ? v : 0.0f);
            } else if (EPI == EPI_FWD_LOGITS) {
                if (a.bias) v += D::ld(static_cast<const T *>(a.bias) + (int64_t)g * a.gBias + n);
                static_cast<float *>(a.C)[ci] = v;
            } else if (EPI == EPI_BWD_DATA) {
                float h = D::ld(static_cast<const T *>(a.mask) + (int64_t)g * a.gMask + (int64_t)m * a.ldm + n);
                static_cast<T *>(a.C)[ci] = D::cvt(h > 0.0f ? v : 0.0f);
            } else {
                T *w = static_cast<T *>(a.C) + ci;
                *w = D::cvt(D::up(*w) - a.lr * v);
            }
        }
    }
}

template <typename D>
static hipError_t launch_typed(int epi, const GemmArgs &a, hipStream_t st)
{
    dim3 grid((unsigned)((a.N + GBN - 1) / GBN), (unsigned)((a.M + GBM - 1) / GBM), (unsigned)a.G);
    dim3 block(256);
    switch (epi) {
    case EPI_FWD_RELU: hipLaunchKernelGGL((k_gemm_generic<D, EPI_FWD_RELU>), grid, block, 0, st, a); break;
    case EPI_FWD_LOGITS: hipLaunchKernelGGL((k_gemm_generic<D, EPI_FWD_LOGITS>), grid, block, 0, st, a); break;
    case EPI_BWD_DATA: hipLaunchKernelGGL((k_gemm_generic<D, EPI_BWD_DATA>), grid, block, 0, st, a); break;
    case EPI_UPDATE: hipLaunchKernelGGL((k_gemm_generic<D, EPI_UPDATE>), grid, block, 0, st, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_gemm_generic(int dtype, int epi, const GemmArgs &a, hipStream_t st)
{
    if (a.M <= 0 || a.N <= 0 || a.G <= 0) return hipSuccess;
    if ((a.M + GBM - 1) / GBM > 65535) return hipErrorInvalidValue;
    return dtype == IST_BF16 ? launch_typed<BF16>(epi, a, st) : launch_typed<F32>(epi, a, st);
}

// IST_GEMM=generic in the environment selects the plain FMA kernel (debugging aid).
static bool force_generic()
{
    static const bool on = [] {
        const char *e = getenv("IST_GEMM");
        return e && std::string(e) == "generic";
    }();
    return on;
}

hipError_t launch_gemm(int dtype, int epi, const GemmArgs &a, hipStream_t st)
{
    return force_generic() ? launch_gemm_generic(dtype, epi, a, st) : launch_gemm_mfma(dtype, epi, a, st);
}

hipError_t launch_gemm_updates(int dtype, const GemmArgs *args, int n, const BiasArgs *bias, bool *bias_done,
                               hipStream_t st)
{
    if (!force_generic()) return launch_gemm_updates_mfma(dtype, args, n, bias, bias_done, st);
    if (bias_done) *bias_done = false;
    for (int i = 0; i < n; ++i) {
        hipError_t e = launch_gemm_generic(dtype, EPI_UPDATE, args[i], st);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

bool gemm_update_shares_launch(int dtype, const GemmArgs &a)
{
    return !force_generic() && gemm_update_shares_launch_mfma(dtype, a);
}

int gemm_splits(int dtype, int epi, const GemmArgs &a)
{
    return force_generic() ? 1 : gemm_splits_mfma(dtype, epi, a);
}

}  // namespace ist
