// Softmax cross-entropy (forward + gradient), loss reduction and bias update of
// the local SGD step (Section 2.1 "Training Subnets"; loss of equation (1) taken
// as the mean softmax cross-entropy over the mini-batch).
#include "ist_internal.h"
#include "ist_bias_block.h"

namespace ist {

__device__ inline float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ inline float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

template <int NT>
__device__ inline float block_reduce(float v, float *sh, bool is_max)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    v = is_max ? wave_max(v) : wave_sum(v);
    __syncthreads();
    if (lane == 0) sh[wave] = v;
    __syncthreads();
    float r = sh[0];
    for (int i = 1; i < NT / 64; ++i) r = is_max ? fmaxf(r, sh[i]) : r + sh[i];
    return r;
}

// One workgroup per (subnet g, sample b): dz = (softmax(z) - onehot(y)) / B in the
// storage dtype, rowloss = logsumexp(z) - z[y].
template <typename D, int NT>
__global__ __launch_bounds__(NT) void k_softmax_xent(const float *__restrict__ logits,
                                                     const int32_t *__restrict__ y,
                                                     int64_t y_stride_g,
                                                     typename D::T *__restrict__ dz,
                                                     float *__restrict__ rowloss, int32_t B,
                                                     int64_t Cn, int64_t ld)
{
    __shared__ float sh[NT / 64];
    const int g = blockIdx.y, b = blockIdx.x;
    const float *z = logits + ((int64_t)g * B + b) * ld;
    typename D::T *out = dz + ((int64_t)g * B + b) * ld;
    float mx = -INFINITY;
    for (int64_t c = threadIdx.x; c < Cn; c += NT) mx = fmaxf(mx, z[c]);
    mx = block_reduce<NT>(mx, sh, true);
    float se = 0.0f;
    for (int64_t c = threadIdx.x; c < Cn; c += NT) se += __expf(z[c] - mx);
    se = block_reduce<NT>(se, sh, false);
    const int32_t label = y[(int64_t)g * y_stride_g + b];
    const float inv = 1.0f / se, invB = 1.0f / (float)B;
    for (int64_t c = threadIdx.x; c < Cn; c += NT) {
        float p = __expf(z[c] - mx) * inv;
        if (c == label) p -= 1.0f;
        out[c] = D::cvt(p * invB);
    }
    if (threadIdx.x == 0) {
        float zl = (label >= 0 && label < Cn) ? z[label] : mx;
        rowloss[(int64_t)g * B + b] = __logf(se) + mx - zl;
    }
}

hipError_t launch_softmax_xent(const float *logits, const int32_t *y, int64_t y_stride_g, void *dz,
                               float *rowloss, int32_t G, int32_t B, int64_t Cn, int64_t ld, int dtype,
                               hipStream_t st)
{
    dim3 grid((unsigned)B, (unsigned)G);
    if (Cn <= 256) {
        if (dtype == IST_BF16)
            hipLaunchKernelGGL((k_softmax_xent<BF16, 64>), grid, dim3(64), 0, st, logits, y, y_stride_g,
                               (uint16_t *)dz, rowloss, B, Cn, ld);
        else
            hipLaunchKernelGGL((k_softmax_xent<F32, 64>), grid, dim3(64), 0, st, logits, y, y_stride_g,
                               (float *)dz, rowloss, B, Cn, ld);
    } else {
        if (dtype == IST_BF16)
            hipLaunchKernelGGL((k_softmax_xent<BF16, 1024>), grid, dim3(1024), 0, st, logits, y,
                               y_stride_g, (uint16_t *)dz, rowloss, B, Cn, ld);
        else
            hipLaunchKernelGGL((k_softmax_xent<F32, 1024>), grid, dim3(1024), 0, st, logits, y,
                               y_stride_g, (float *)dz, rowloss, B, Cn, ld);
    }
    return hipGetLastError();
}

// Narrow output layer (Cn <= 256): one wave per (subnet g, sample b), four per workgroup, the
// classes lane, lane + 64, ... of the row in registers.  The logits are either stored values
// (splits == 1, bias already added) or the sum, in split order, of the fp32 partial products
// of a k-split forward product plus the bias, so that such a product needs no finishing pass.
template <typename D>
__global__ __launch_bounds__(256) void k_xent_rows(const float *__restrict__ z, int32_t splits, int64_t split_stride,
                                                   int64_t g_stride, int64_t ldz,
                                                   const typename D::T *__restrict__ bias, int64_t gBias,
                                                   const int32_t *__restrict__ y, int64_t y_stride_g,
                                                   typename D::T *__restrict__ dz, int64_t ld,
                                                   float *__restrict__ rowloss, int32_t G, int32_t B, int32_t Cn,
                                                   float alpha)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= (int64_t)G * B) return;
    const int g = (int)(row / B), b = (int)(row % B);
    const float *zr = z + (int64_t)g * g_stride + (int64_t)b * ldz;
    float v[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int c = lane + 64 * i;
        float acc = 0.0f;
        if (c < Cn) {
#pragma unroll 8
            for (int sp = 0; sp < splits; ++sp) acc += zr[(int64_t)sp * split_stride + c];
            acc *= alpha;
            if (bias) acc += D::ld(bias + (int64_t)g * gBias + c);
        }
        v[i] = c < Cn ? acc : -INFINITY;
    }
    const int32_t label = y[(int64_t)g * y_stride_g + b];
    const float mx = wave_max(fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3])));
    float e[4], se = 0.0f, zl = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int c = lane + 64 * i;
        e[i] = c < Cn ? __expf(v[i] - mx) : 0.0f;
        se += e[i];
        zl += (c < Cn && c == label) ? v[i] : 0.0f;
    }
    se = wave_sum(se);
    zl = wave_sum(zl);
    const float inv = 1.0f / se, invB = 1.0f / (float)B;
    typename D::T *out = dz + ((int64_t)g * B + b) * ld;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int c = lane + 64 * i;
        if (c < Cn) out[c] = D::cvt((e[i] * inv - (c == label ? 1.0f : 0.0f)) * invB);
    }
    if (lane == 0) rowloss[row] = __logf(se) + mx - ((label >= 0 && label < Cn) ? zl : mx);
}

hipError_t launch_xent_rows(const float *z, int32_t splits, int64_t split_stride, int64_t g_stride, int64_t ldz,
                            const void *bias, int64_t gBias, const int32_t *y, int64_t y_stride_g, void *dz,
                            int64_t ld, float *rowloss, int32_t G, int32_t B, int32_t Cn, int dtype, hipStream_t st,
                            float alpha)
{
    if (Cn > 256 || splits < 1) return hipErrorInvalidValue;
    const dim3 grid((unsigned)(((int64_t)G * B + 3) / 4));
    if (dtype == IST_BF16)
        hipLaunchKernelGGL((k_xent_rows<BF16>), grid, dim3(256), 0, st, z, splits, split_stride, g_stride, ldz,
                           static_cast<const uint16_t *>(bias), gBias, y, y_stride_g, static_cast<uint16_t *>(dz), ld,
                           rowloss, G, B, Cn, alpha);
    else
        hipLaunchKernelGGL((k_xent_rows<F32>), grid, dim3(256), 0, st, z, splits, split_stride, g_stride, ldz,
                           static_cast<const float *>(bias), gBias, y, y_stride_g, static_cast<float *>(dz), ld,
                           rowloss, G, B, Cn, alpha);
    return hipGetLastError();
}

// loss_out[g * out_stride_g + j] = mean_b rowloss[j][g][b] for the steps j < nsteps of a call whose
// row losses are still waiting; one wave per (subnet, step), fixed order.
__global__ __launch_bounds__(64) void k_loss_reduce(const float *__restrict__ rowloss,
                                                    float *__restrict__ loss_out,
                                                    int64_t out_stride_g, int32_t G, int32_t B)
{
    const int g = blockIdx.x, j = blockIdx.y;
    const float *r = rowloss + ((int64_t)j * G + g) * B;
    float acc = 0.0f;
    for (int b = threadIdx.x; b < B; b += 64) acc += r[b];
    acc = wave_sum(acc);
    if (threadIdx.x == 0) loss_out[(int64_t)g * out_stride_g + j] = acc / (float)B;
}

hipError_t launch_loss_reduce(const float *rowloss, float *loss_out, int64_t out_stride_g, int32_t G,
                              int32_t B, int32_t nsteps, hipStream_t st)
{
    hipLaunchKernelGGL(k_loss_reduce, dim3((unsigned)G, (unsigned)nsteps), dim3(64), 0, st, rowloss, loss_out,
                       out_stride_g, G, B);
    return hipGetLastError();
}

// Row statistics of a wide output layer from the per-column-block partials of the
// forward pass (layout [g][block][row]): two levels of the usual (max, sum) merge,
// lse = log sum_blocks psum * exp(pmax - max) + max, loss = lse - z[label].
constexpr int kLseChunks = 32;

__device__ inline void lse_merge(float &m, float &s, float m2, float s2)
{
    const float mx = fmaxf(m, m2);
    if (mx == -INFINITY) { m = mx; s = 0.0f; return; }
    s = s * __expf(m - mx) + s2 * __expf(m2 - mx);
    m = mx;
}

// level 1: workgroup = 64 rows x 4 waves; wave w takes blocks c0 + w, c0 + w + 4, ... of chunk c
__global__ __launch_bounds__(256) void k_lse_level1(const float *__restrict__ pmax,
                                                    const float *__restrict__ psum, int32_t nb, int32_t M,
                                                    float *__restrict__ qmax, float *__restrict__ qsum)
{
    __shared__ float shm[4][64], shs[4][64];
    const int g = blockIdx.z, c = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row = blockIdx.x * 64 + lane;
    const int per = (nb + kLseChunks - 1) / kLseChunks;
    const int b0 = c * per, b1 = min(nb, b0 + per);
    float m = -INFINITY, s = 0.0f;
    if (row < M) {
        for (int b = b0 + wave; b < b1; b += 4) {
            const int64_t i = ((int64_t)g * nb + b) * M + row;
            lse_merge(m, s, pmax[i], psum[i]);
        }
    }
    shm[wave][lane] = m; shs[wave][lane] = s;
    __syncthreads();
    if (wave == 0 && row < M) {
        for (int w = 1; w < 4; ++w) lse_merge(m, s, shm[w][lane], shs[w][lane]);
        const int64_t o = ((int64_t)g * kLseChunks + c) * M + row;
        qmax[o] = m; qsum[o] = s;
    }
}

__global__ __launch_bounds__(256) void k_lse_level2(const float *__restrict__ qmax,
                                                    const float *__restrict__ qsum, int32_t M,
                                                    const float *__restrict__ zlabel,
                                                    const int32_t *__restrict__ y, int64_t gY, int64_t Cn,
                                                    float *__restrict__ lse, float *__restrict__ rowloss)
{
    const int g = blockIdx.y;
    const int row = blockIdx.x * 256 + threadIdx.x;
    if (row >= M) return;
    float m = -INFINITY, s = 0.0f;
    for (int c = 0; c < kLseChunks; ++c) {
        const int64_t i = ((int64_t)g * kLseChunks + c) * M + row;
        lse_merge(m, s, qmax[i], qsum[i]);
    }
    const float l = __logf(s) + m;
    const int64_t r = (int64_t)g * M + row;
    lse[r] = l;
    const int32_t label = y[(int64_t)g * gY + row];
    rowloss[r] = (label >= 0 && label < Cn) ? l - zlabel[r] : 0.0f;
}

hipError_t launch_lse_combine(const float *pmax, const float *psum, int32_t nb, float *qmax, float *qsum,
                              const float *zlabel, const int32_t *y, int64_t gY, int64_t Cn, float *lse,
                              float *rowloss, int32_t G, int32_t B, hipStream_t st)
{
    hipLaunchKernelGGL(k_lse_level1, dim3((unsigned)((B + 63) / 64), kLseChunks, (unsigned)G), dim3(256), 0, st, pmax,
                       psum, nb, B, qmax, qsum);
    hipLaunchKernelGGL(k_lse_level2, dim3((unsigned)((B + 255) / 256), (unsigned)G), dim3(256), 0, st, qmax, qsum, B,
                       zlabel, y, gY, Cn, lse, rowloss);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Per-neuron standardisation over the mini-batch (Section 2.2 "Correcting Distributional
// Shift"; no learned scale or shift, statistics of the current batch, fp32 arithmetic).
// A workgroup owns 64 columns of one subnet; its 4 wavefronts split the batch rows
// (row b goes to wave b % 4, ascending), partial sums meet in LDS in fixed order.
// ---------------------------------------------------------------------------------------
__device__ inline float col_reduce4(float v, float (*sh)[64], int wave, int lane)
{
    __syncthreads();
    sh[wave][lane] = v;
    __syncthreads();
    return (sh[0][lane] + sh[1][lane]) + (sh[2][lane] + sh[3][lane]);
}

template <typename D>
__global__ __launch_bounds__(256) void k_norm_forward(const float *__restrict__ z, typename D::T *__restrict__ zh,
                                                      typename D::T *__restrict__ h, float *__restrict__ isg,
                                                      int32_t B, int64_t R, int64_t ld, float eps)
{
    using T = typename D::T;
    __shared__ float sh[4][64];
    const int g = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t r = (int64_t)blockIdx.x * 64 + lane;
    const bool ok = r < R;
    const int64_t base = (int64_t)g * B * ld + (ok ? r : 0);
    const float invB = 1.0f / (float)B;
    float acc = 0.0f;
    for (int b = wave; b < B; b += 4) acc += ok ? z[base + (int64_t)b * ld] : 0.0f;
    const float mu = col_reduce4(acc, sh, wave, lane) * invB;
    acc = 0.0f;
    for (int b = wave; b < B; b += 4) {
        const float d = (ok ? z[base + (int64_t)b * ld] : mu) - mu;
        acc = fmaf(d, d, acc);
    }
    const float var = col_reduce4(acc, sh, wave, lane) * invB;
    const float inv = 1.0f / sqrtf(var + eps);
    if (!ok) return;
    if (wave == 0) isg[(int64_t)g * ld + r] = inv;
    for (int b = wave; b < B; b += 4) {
        const T v = D::cvt((z[base + (int64_t)b * ld] - mu) * inv);
        zh[base + (int64_t)b * ld] = v;
        h[base + (int64_t)b * ld] = D::up(v) > 0.0f ? v : D::cvt(0.0f);
    }
}

template <typename D>
__global__ __launch_bounds__(256) void k_norm_backward(typename D::T *__restrict__ dz,
                                                       const typename D::T *__restrict__ zh,
                                                       const float *__restrict__ isg, int32_t B, int64_t R, int64_t ld)
{
    __shared__ float sh[4][64];
    const int g = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t r = (int64_t)blockIdx.x * 64 + lane;
    const bool ok = r < R;
    const int64_t base = (int64_t)g * B * ld + (ok ? r : 0);
    const float invB = 1.0f / (float)B;
    float a1 = 0.0f, a2 = 0.0f;
    for (int b = wave; b < B; b += 4) {
        const float d = ok ? D::ld(dz + base + (int64_t)b * ld) : 0.0f;
        const float v = ok ? D::ld(zh + base + (int64_t)b * ld) : 0.0f;
        a1 += d;
        a2 = fmaf(d, v, a2);
    }
    const float s1 = col_reduce4(a1, sh, wave, lane) * invB;
    const float s2 = col_reduce4(a2, sh, wave, lane) * invB;
    if (!ok) return;
    const float inv = isg[(int64_t)g * ld + r];
    for (int b = wave; b < B; b += 4) {
        const float d = D::ld(dz + base + (int64_t)b * ld);
        const float v = D::ld(zh + base + (int64_t)b * ld);
        dz[base + (int64_t)b * ld] = D::cvt((d - s1 - v * s2) * inv);
    }
}

// Batches of up to 512 rows: 16 wavefronts per workgroup, every thread keeps its (at most 32) rows of
// the column in registers, so the pre-activations are read once and all loads are in flight together.
constexpr int kNormWaves = 16, kNormRows = 32;

__device__ inline float col_reduce16(float v, float (*sh)[64], int wave, int lane)
{
    __syncthreads();
    sh[wave][lane] = v;
    __syncthreads();
    float t[kNormWaves];
#pragma unroll
    for (int i = 0; i < kNormWaves; ++i) t[i] = sh[i][lane];
#pragma unroll
    for (int d = 1; d < kNormWaves; d *= 2)
#pragma unroll
        for (int i = 0; i + d < kNormWaves; i += 2 * d) t[i] += t[i + d];
    return t[0];
}

template <typename D>
__global__ __launch_bounds__(64 * kNormWaves) void k_norm_forward_reg(const float *__restrict__ z,
                                                                      typename D::T *__restrict__ zh,
                                                                      typename D::T *__restrict__ h,
                                                                      float *__restrict__ isg, int32_t B, int64_t R,
                                                                      int64_t ld, float eps)
{
    using T = typename D::T;
    __shared__ float sh[kNormWaves][64];
    const int g = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t r = (int64_t)blockIdx.x * 64 + lane;
    const bool ok = r < R;
    const int64_t base = (int64_t)g * B * ld + (ok ? r : 0);
    const float invB = 1.0f / (float)B;
    float v[kNormRows];
#pragma unroll
    for (int i = 0; i < kNormRows; ++i) {
        const int b = wave + kNormWaves * i;
        v[i] = (ok && b < B) ? z[base + (int64_t)b * ld] : 0.0f;
    }
    float acc = 0.0f;
#pragma unroll
    for (int i = 0; i < kNormRows; ++i) acc += v[i];
    const float mu = col_reduce16(acc, sh, wave, lane) * invB;
    acc = 0.0f;
#pragma unroll
    for (int i = 0; i < kNormRows; ++i) {
        const float d = (wave + kNormWaves * i < B) ? v[i] - mu : 0.0f;
        acc = fmaf(d, d, acc);
    }
    const float var = col_reduce16(acc, sh, wave, lane) * invB;
    const float inv = 1.0f / sqrtf(var + eps);
    if (!ok) return;
    if (wave == 0) isg[(int64_t)g * ld + r] = inv;
#pragma unroll
    for (int i = 0; i < kNormRows; ++i) {
        const int b = wave + kNormWaves * i;
        if (b < B) {
            const T q = D::cvt((v[i] - mu) * inv);
            zh[base + (int64_t)b * ld] = q;
            h[base + (int64_t)b * ld] = D::up(q) > 0.0f ? q : D::cvt(0.0f);
        }
    }
}

template <typename D>
__global__ __launch_bounds__(64 * kNormWaves) void k_norm_backward_reg(typename D::T *__restrict__ dz,
                                                                       const typename D::T *__restrict__ zh,
                                                                       const float *__restrict__ isg, int32_t B,
                                                                       int64_t R, int64_t ld)
{
    __shared__ float sh[kNormWaves][64];
    const int g = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t r = (int64_t)blockIdx.x * 64 + lane;
    const bool ok = r < R;
    const int64_t base = (int64_t)g * B * ld + (ok ? r : 0);
    const float invB = 1.0f / (float)B;
    float d[kNormRows], v[kNormRows];
#pragma unroll
    for (int i = 0; i < kNormRows; ++i) {
        const int b = wave + kNormWaves * i;
        const bool in = ok && b < B;
        d[i] = in ? D::ld(dz + base + (int64_t)b * ld) : 0.0f;
        v[i] = in ? D::ld(zh + base + (int64_t)b * ld) : 0.0f;
    }
    float a1 = 0.0f, a2 = 0.0f;
#pragma unroll
    for (int i = 0; i < kNormRows; ++i) { a1 += d[i]; a2 = fmaf(d[i], v[i], a2); }
    const float s1 = col_reduce16(a1, sh, wave, lane) * invB;
    const float s2 = col_reduce16(a2, sh, wave, lane) * invB;
    if (!ok) return;
    const float inv = isg[(int64_t)g * ld + r];
#pragma unroll
    for (int i = 0; i < kNormRows; ++i) {
        const int b = wave + kNormWaves * i;
        if (b < B) dz[base + (int64_t)b * ld] = D::cvt((d[i] - s1 - v[i] * s2) * inv);
    }
}

// bf16 layers at least 2048 wide: two neighbouring columns per lane (8-byte loads of z, 4-byte packed
// accesses of the bf16 arrays), 128 columns per workgroup.  Needs an even pitch (it is a multiple of 8).
__global__ __launch_bounds__(64 * kNormWaves) void k_norm_forward_bf16x2(const float *__restrict__ z,
                                                                         uint32_t *__restrict__ zh,
                                                                         uint32_t *__restrict__ h,
                                                                         float *__restrict__ isg, int32_t B, int64_t R,
                                                                         int64_t ld, float eps)
{
    __shared__ float sh[kNormWaves][64];
    const int g = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t r = ((int64_t)blockIdx.x * 64 + lane) * 2;   // r even, ld even: r + 1 < ld whenever r < R
    const bool ok = r < R;
    const int64_t base = (int64_t)g * B * ld + (ok ? r : 0);
    const float invB = 1.0f / (float)B;
    float2 v[kNormRows];
#pragma unroll
    for (int i = 0; i < kNormRows; ++i) {
        const int b = wave + kNormWaves * i;
        v[i] = (ok && b < B) ? *reinterpret_cast<const float2 *>(z + base + (int64_t)b * ld) : float2{0.0f, 0.0f};
    }
    float a0 = 0.0f, a1 = 0.0f;
#pragma unroll
    for (int i = 0; i < kNormRows; ++i) { a0 += v[i].x; a1 += v[i].y; }
    const float mu0 = col_reduce16(a0, sh, wave, lane) * invB;
    const float mu1 = col_reduce16(a1, sh, wave, lane) * invB;
    a0 = a1 = 0.0f;
#pragma unroll
    for (int i = 0; i < kNormRows; ++i) {
        const bool in = wave + kNormWaves * i < B;
        const float d0 = in ? v[i].x - mu0 : 0.0f, d1 = in ? v[i].y - mu1 : 0.0f;
        a0 = fmaf(d0, d0, a0);
        a1 = fmaf(d1, d1, a1);
    }
    const float inv0 = 1.0f / sqrtf(col_reduce16(a0, sh, wave, lane) * invB + eps);
    const float inv1 = 1.0f / sqrtf(col_reduce16(a1, sh, wave, lane) * invB + eps);
    if (!ok) return;
    if (wave == 0) { isg[(int64_t)g * ld + r] = inv0; isg[(int64_t)g * ld + r + 1] = inv1; }
#pragma unroll
    for (int i = 0; i < kNormRows; ++i) {
        const int b = wave + kNormWaves * i;
        if (b < B) {
            const uint32_t q = f32x2_to_bf16x2((v[i].x - mu0) * inv0, (v[i].y - mu1) * inv1);
            const uint32_t lo = (q & 0x8000u) || !(q & 0x7fffu) ? 0u : (q & 0xffffu);          // max(. , 0) per half
            const uint32_t hi = (q & 0x80000000u) || !(q & 0x7fff0000u) ? 0u : (q & 0xffff0000u);
            zh[(base + (int64_t)b * ld) >> 1] = q;
            h[(base + (int64_t)b * ld) >> 1] = lo | hi;
        }
    }
}

__global__ __launch_bounds__(64 * kNormWaves) void k_norm_backward_bf16x2(uint32_t *__restrict__ dz,
                                                                          const uint32_t *__restrict__ zh,
                                                                          const float *__restrict__ isg, int32_t B,
                                                                          int64_t R, int64_t ld)
{
    __shared__ float sh[kNormWaves][64];
    const int g = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t r = ((int64_t)blockIdx.x * 64 + lane) * 2;
    const bool ok = r < R;
    const int64_t base = (int64_t)g * B * ld + (ok ? r : 0);
    const float invB = 1.0f / (float)B;
    uint32_t d[kNormRows], v[kNormRows];
#pragma unroll
    for (int i = 0; i < kNormRows; ++i) {
        const int b = wave + kNormWaves * i;
        const bool in = ok && b < B;
        d[i] = in ? dz[(base + (int64_t)b * ld) >> 1] : 0u;
        v[i] = in ? zh[(base + (int64_t)b * ld) >> 1] : 0u;
    }
    auto lo = [](uint32_t x) { return __uint_as_float(x << 16); };
    auto hi = [](uint32_t x) { return __uint_as_float(x & 0xffff0000u); };
    float p0 = 0.0f, p1 = 0.0f, q0 = 0.0f, q1 = 0.0f;
#pragma unroll
    for (int i = 0; i < kNormRows; ++i) {
        p0 += lo(d[i]); p1 += hi(d[i]);
        q0 = fmaf(lo(d[i]), lo(v[i]), q0);
        q1 = fmaf(hi(d[i]), hi(v[i]), q1);
    }
    const float s10 = col_reduce16(p0, sh, wave, lane) * invB, s11 = col_reduce16(p1, sh, wave, lane) * invB;
    const float s20 = col_reduce16(q0, sh, wave, lane) * invB, s21 = col_reduce16(q1, sh, wave, lane) * invB;
    if (!ok) return;
    const float inv0 = isg[(int64_t)g * ld + r], inv1 = isg[(int64_t)g * ld + r + 1];
#pragma unroll
    for (int i = 0; i < kNormRows; ++i) {
        const int b = wave + kNormWaves * i;
        if (b < B)
            dz[(base + (int64_t)b * ld) >> 1] = f32x2_to_bf16x2((lo(d[i]) - s10 - lo(v[i]) * s20) * inv0,
                                                                (hi(d[i]) - s11 - hi(v[i]) * s21) * inv1);
    }
}

static bool norm_pairs_ok(const void *a, const void *b, int64_t R, int64_t ld, int32_t B, int dtype)
{
    return dtype == IST_BF16 && R >= 2048 && ld % 2 == 0 && ((int64_t)B * ld) % 2 == 0 &&
           reinterpret_cast<uintptr_t>(a) % 8 == 0 && reinterpret_cast<uintptr_t>(b) % 8 == 0;
}

hipError_t launch_norm_forward(const float *z, void *zh, void *h, float *isg, int32_t G, int32_t B, int64_t R,
                               int64_t ld, float eps, int dtype, hipStream_t st)
{
    const dim3 grid((unsigned)((R + 63) / 64), (unsigned)G);
    if (B <= kNormWaves * kNormRows && norm_pairs_ok(z, zh, R, ld, B, dtype) && reinterpret_cast<uintptr_t>(h) % 8 == 0) {
        hipLaunchKernelGGL(k_norm_forward_bf16x2, dim3((unsigned)((R + 127) / 128), (unsigned)G), dim3(64 * kNormWaves), 0, st,
                           z, (uint32_t *)zh, (uint32_t *)h, isg, B, R, ld, eps);
        return hipGetLastError();
    }
    if (B <= kNormWaves * kNormRows) {
        if (dtype == IST_BF16)
            hipLaunchKernelGGL(k_norm_forward_reg<BF16>, grid, dim3(64 * kNormWaves), 0, st, z, (uint16_t *)zh, (uint16_t *)h,
                               isg, B, R, ld, eps);
        else
            hipLaunchKernelGGL(k_norm_forward_reg<F32>, grid, dim3(64 * kNormWaves), 0, st, z, (float *)zh, (float *)h, isg, B,
                               R, ld, eps);
        return hipGetLastError();
    }
    if (dtype == IST_BF16)
        hipLaunchKernelGGL(k_norm_forward<BF16>, grid, dim3(256), 0, st, z, (uint16_t *)zh, (uint16_t *)h, isg, B, R, ld, eps);
    else
        hipLaunchKernelGGL(k_norm_forward<F32>, grid, dim3(256), 0, st, z, (float *)zh, (float *)h, isg, B, R, ld, eps);
    return hipGetLastError();
}

hipError_t launch_norm_backward(void *dz, const void *zh, const float *isg, int32_t G, int32_t B, int64_t R,
                                int64_t ld, int dtype, hipStream_t st)
{
    const dim3 grid((unsigned)((R + 63) / 64), (unsigned)G);
    if (B <= kNormWaves * kNormRows && norm_pairs_ok(dz, zh, R, ld, B, dtype)) {
        hipLaunchKernelGGL(k_norm_backward_bf16x2, dim3((unsigned)((R + 127) / 128), (unsigned)G), dim3(64 * kNormWaves), 0, st,
                           (uint32_t *)dz, (const uint32_t *)zh, isg, B, R, ld);
        return hipGetLastError();
    }
    if (B <= kNormWaves * kNormRows) {
        if (dtype == IST_BF16)
            hipLaunchKernelGGL(k_norm_backward_reg<BF16>, grid, dim3(64 * kNormWaves), 0, st, (uint16_t *)dz,
                               (const uint16_t *)zh, isg, B, R, ld);
        else
            hipLaunchKernelGGL(k_norm_backward_reg<F32>, grid, dim3(64 * kNormWaves), 0, st, (float *)dz, (const float *)zh,
                               isg, B, R, ld);
        return hipGetLastError();
    }
    if (dtype == IST_BF16)
        hipLaunchKernelGGL(k_norm_backward<BF16>, grid, dim3(256), 0, st, (uint16_t *)dz, (const uint16_t *)zh, isg, B, R, ld);
    else
        hipLaunchKernelGGL(k_norm_backward<F32>, grid, dim3(256), 0, st, (float *)dz, (const float *)zh, isg, B, R, ld);
    return hipGetLastError();
}

template <typename D>
__global__ __launch_bounds__(256) void k_bias_update(BiasArgs a)
{
    bias_update_block<D>(a, (int)blockIdx.x, (int)blockIdx.y);
}

// Wide layers: a workgroup owns 512 columns (8 per lane, one 16-byte load per lane and row), its
// 4 wavefronts split the batch rows and keep 4 rows in flight each.  Needs a 16-byte aligned
// dz with a pitch that is a multiple of 8 elements (bf16) / 4 (f32: two loads per row).
// All wide layers of a step share one launch (blockIdx.z = layer): a single layer's 512-column blocks
// leave half of the chip idle.
template <typename D>
__global__ __launch_bounds__(256) void k_bias_update_wide(BiasArgs a)
{
    using T = typename D::T;
    constexpr int V = 8;                       // columns per lane
    constexpr int NV = V * sizeof(T) / 16;     // 16-byte loads per lane and row
    __shared__ float part[3][64][V + 1];
    const BiasJob jb = a.job[blockIdx.z];
    const int32_t B = a.B;
    const float lr = a.lr;
    if ((int64_t)blockIdx.x * 512 >= jb.ld) return;   // (a whole workgroup: the barrier below is safe)
    const int g = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t c0 = ((int64_t)blockIdx.x * 64 + lane) * V;
    float acc[V];
#pragma unroll
    for (int i = 0; i < V; ++i) acc[i] = 0.0f;
    if (c0 < jb.ld) {   // the padding columns of a row are zero and are not stored below
        const T *p = static_cast<const T *>(jb.dz) + (int64_t)g * B * jb.ld + c0;
        auto add = [&](const uint4 (&r)[NV]) {
            if (sizeof(T) == 2) {
                const uint32_t w[4] = {r[0].x, r[0].y, r[0].z, r[0].w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    acc[2 * i] += __uint_as_float(w[i] << 16);
                    acc[2 * i + 1] += __uint_as_float(w[i] & 0xffff0000u);
                }
            } else {
#pragma unroll
                for (int v = 0; v < NV; ++v) {
                    acc[4 * v] += __uint_as_float(r[v].x); acc[4 * v + 1] += __uint_as_float(r[v].y);
                    acc[4 * v + 2] += __uint_as_float(r[v].z); acc[4 * v + 3] += __uint_as_float(r[v].w);
                }
            }
        };
        int b = wave;
        for (; b + 12 < B; b += 16) {
            uint4 r[4][NV];
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int v = 0; v < NV; ++v)
                    r[u][v] = reinterpret_cast<const uint4 *>(p + (int64_t)(b + 4 * u) * jb.ld)[v];
#pragma unroll
            for (int u = 0; u < 4; ++u) add(r[u]);
        }
        for (; b < B; b += 4) {
            uint4 r[NV];
#pragma unroll
            for (int v = 0; v < NV; ++v) r[v] = reinterpret_cast<const uint4 *>(p + (int64_t)b * jb.ld)[v];
            add(r);
        }
    }
    if (wave > 0) {
#pragma unroll
        for (int i = 0; i < V; ++i) part[wave - 1][lane][i] = acc[i];
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
        for (int i = 0; i < V; ++i) {
            const float tot = (acc[i] + part[0][lane][i]) + (part[1][lane][i] + part[2][lane][i]);
            if (c0 + i < jb.R) {
                T *w = static_cast<T *>(jb.bias) + (int64_t)g * jb.R + c0 + i;
                *w = D::cvt(D::up(*w) - lr * tot);
            }
        }
    }
}

// Bias update of a wide output layer from the per-class partial sums that the dz pass left:
// bias[g][r] -= lr * sum_blk rsum[(g * nrb + blk) * R + r], blocks in ascending order.
template <typename D>
__global__ __launch_bounds__(256) void k_bias_apply(typename D::T *__restrict__ bias, const float *__restrict__ rsum,
                                                    int32_t nrb, int64_t R, float lr)
{
    const int g = blockIdx.y;
    const int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (r >= R) return;
    float acc = 0.0f;
    for (int blk = 0; blk < nrb; ++blk) acc += rsum[((int64_t)g * nrb + blk) * R + r];
    typename D::T *b = bias + (int64_t)g * R + r;
    *b = D::cvt(D::ld(b) - lr * acc);
}

hipError_t launch_bias_apply(void *bias, const float *rsum, int32_t nrb, int64_t R, int32_t G, float lr, int dtype,
                             hipStream_t st)
{
    dim3 grid((unsigned)((R + 255) / 256), (unsigned)G);
    if (dtype == IST_BF16)
        hipLaunchKernelGGL(k_bias_apply<BF16>, grid, dim3(256), 0, st, static_cast<uint16_t *>(bias), rsum, nrb, R, lr);
    else
        hipLaunchKernelGGL(k_bias_apply<F32>, grid, dim3(256), 0, st, static_cast<float *>(bias), rsum, nrb, R, lr);
    return hipGetLastError();
}

static bool bias_job_wide(const BiasJob &jb, int32_t B, int dtype)
{
    const int che = dtype == IST_BF16 ? 8 : 4;
    return jb.R >= 2048 && jb.ld % 8 == 0 && reinterpret_cast<uintptr_t>(jb.dz) % 16 == 0 && ((int64_t)B * jb.ld) % che == 0;
}

bool bias_jobs_all_narrow(const BiasArgs &a, int dtype)
{
    for (int j = 0; j < a.njobs; ++j)
        if (bias_job_wide(a.job[j], a.B, dtype)) return false;
    return true;
}

hipError_t launch_bias_update(BiasArgs &a, int dtype, hipStream_t st)
{
    if (a.njobs <= 0) return hipSuccess;
    // wide layers go to the 16-byte kernel (one launch for all of them); the rest share another launch
    BiasArgs wide = a;
    wide.njobs = 0;
    int kept = 0;
    int64_t widest = 0;
    for (int j = 0; j < a.njobs; ++j) {
        const BiasJob &jb = a.job[j];
        if (!bias_job_wide(jb, a.B, dtype)) { a.job[kept++] = jb; continue; }
        wide.job[wide.njobs++] = jb;
        widest = jb.ld > widest ? jb.ld : widest;
    }
    if (wide.njobs > 0) {
        dim3 grid((unsigned)((widest + 511) / 512), (unsigned)a.G, (unsigned)wide.njobs);
        if (dtype == IST_BF16)
            hipLaunchKernelGGL(k_bias_update_wide<BF16>, grid, dim3(256), 0, st, wide);
        else
            hipLaunchKernelGGL(k_bias_update_wide<F32>, grid, dim3(256), 0, st, wide);
    }
    a.njobs = kept;
    if (a.njobs <= 0) return hipGetLastError();
    int blocks = 0;
    for (int j = 0; j < a.njobs; ++j) {
        a.job[j].blk0 = blocks;
        blocks += (int)((a.job[j].R + 63) / 64);
    }
    dim3 grid((unsigned)blocks, (unsigned)a.G);
    if (dtype == IST_BF16)
        hipLaunchKernelGGL(k_bias_update<BF16>, grid, dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL(k_bias_update<F32>, grid, dim3(256), 0, st, a);
    return hipGetLastError();
}

}  // namespace ist
