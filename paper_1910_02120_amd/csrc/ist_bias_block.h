// Bias update of narrow layers, as a block-level routine shared by the stand-alone kernel and by the
// launch that carries the update products of several layers.
#pragma once
#include "ist_internal.h"

namespace ist {

// b_l[g][r] <- b_l[g][r] - lr * sum_b dz_l[g][b][r] for several layers in one launch.
// A workgroup (256 threads) owns 64 columns of one (layer, subnet): block blk of the jobs' concatenated
// column blocks, subnet g; its 4 wavefronts split the batch rows, partial sums meet in LDS, summation
// order is fixed.
template <typename D>
__device__ inline void bias_update_block(const BiasArgs &a, int blk, int g)
{
    using T = typename D::T;
    __shared__ float part[4][64];
    int j = 0;
    while (j + 1 < a.njobs && blk >= a.job[j + 1].blk0) ++j;
    const BiasJob jb = a.job[j];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t r = (int64_t)(blk - jb.blk0) * 64 + lane;
    float acc = 0.0f;
    if (r < jb.R) {
        const T *p = static_cast<const T *>(jb.dz) + (int64_t)g * a.B * jb.ld + r;
        int b = wave;
        for (; b + 28 < a.B; b += 32) {   // 8 rows in flight per wave; the order of the sum stays b ascending
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = D::ld(p + (int64_t)(b + 4 * u) * jb.ld);
#pragma unroll
            for (int u = 0; u < 8; ++u) acc += v[u];
        }
        for (; b < a.B; b += 4) acc += D::ld(p + (int64_t)b * jb.ld);
    }
    part[wave][lane] = acc;
    __syncthreads();
    if (wave == 0 && r < jb.R) {
        float tot = (part[0][lane] + part[1][lane]) + (part[2][lane] + part[3][lane]);
        T *w = static_cast<T *>(jb.bias) + (int64_t)g * jb.R + r;
        *w = D::cvt(D::up(*w) - a.lr * tot);
    }
}

}  // namespace ist
