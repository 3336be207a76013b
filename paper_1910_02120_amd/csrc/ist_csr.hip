// Sparse-input first layer (the extreme-classification workload of Section 3.1:
// 135,909 sparse features).  The subnet's W_1 block is stored transposed,
// Wt[g][c][q] = W_1[H_1^g[q]][c], so that one non-zero of a sample touches one
// contiguous row of w = N_1/S values.
//
//   forward : h_1[b][q] = ReLU(sum_{(c,v) in row b} v * Wt[c][q] + b_1[q])
//   update  : Wt[c][:] <- Wt[c][:] - lr * sum_{b : c in row b} x[b][c] * dz_1[b][:]
//             for the columns c that occur in the batch (all others have a zero
//             gradient).  The sum over b runs in ascending b so the result does not
//             depend on scheduling: a bitmap (one bit per sample) per column is
//             built with integer atomics, then one wavefront owns one column.
#include <algorithm>

#include "ist_internal.h"

namespace ist {

// ROWMAJOR: Wt is an untransposed W_1 [w][N0] instead (the full network's first layer: one group,
// strided weight reads - an evaluation path, not the training one).
template <typename D, bool ROWMAJOR = false>
__global__ __launch_bounds__(256) void k_csr_forward(CsrArgs c, const typename D::T *__restrict__ Wt,
                                                     const typename D::T *__restrict__ bias,
                                                     typename D::T *__restrict__ h, float *__restrict__ z_out)
{
    using T = typename D::T;
    const int g = blockIdx.z, b = blockIdx.y;
    const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= c.w) return;
    const int64_t row = c.row0 + (int64_t)g * c.stride_g + b;
    int64_t p0 = c.rowptr[row], p1 = c.rowptr[row + 1];
    p0 = p0 < 0 ? 0 : p0;
    p1 = p1 > c.nnz ? c.nnz : p1;
    const T *Wg = Wt + (int64_t)g * c.N0 * c.w;
    const T *vals = static_cast<const T *>(c.vals);
    float acc = 0.0f;
    for (int64_t p = p0; p < p1; ++p) {
        int32_t col = c.colidx[p];
        if (col < 0 || col >= c.N0) continue;
        acc = fmaf(D::up(vals[p]), D::ld(ROWMAJOR ? Wg + q * c.N0 + col : Wg + (int64_t)col * c.w + q), acc);
    }
    acc *= c.alpha;
    if (bias) acc += D::ld(bias + (int64_t)g * c.w + q);
    if (z_out) z_out[((int64_t)g * c.B + b) * c.ld + q] = acc;
    else h[((int64_t)g * c.B + b) * c.ld + q] = D::cvt(acc > 0.0f ? acc : 0.0f);
}

__global__ void k_fill_u32(uint32_t *p, int64_t n, uint32_t v)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * blockDim.x)
        p[i] = v;
}

hipError_t launch_fill_u32(void *p, int64_t n, uint32_t v, hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    const unsigned blocks = (unsigned)std::min<int64_t>(2048, (n + 255) / 256);
    hipLaunchKernelGGL(k_fill_u32, dim3(blocks), dim3(256), 0, st, static_cast<uint32_t *>(p), n, v);
    return hipGetLastError();
}

hipError_t launch_fill_zero(void *p, size_t bytes, hipStream_t st)
{
    return launch_fill_u32(p, (int64_t)(bytes / 4), 0u, st);
}

// Scratch of the sparse update, per (group, column): `words` bitmap words (one bit per sample), and after all of
// them one 64-bit word per pair that names the column's first occurrence in the batch.
__host__ __device__ inline int64_t csr_bitmap_words(int64_t G, int64_t N0, int words) { return (G * N0 * words + 1) / 2 * 2; }
size_t csr_scratch_bytes(int64_t G, int64_t N0, int64_t B)
{
    return (size_t)csr_bitmap_words(G, N0, (int)((B + 31) / 32)) * 4 + (size_t)G * N0 * 8;
}
constexpr uint64_t kPosMask = (1ull << 40) - 1;   // first[] = ((sample << 40) | position in vals) + 1; 0: look it up

__global__ void k_csr_clear(uint32_t *bitmap, int64_t nwords, uint64_t *first, int64_t npairs)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nwords; i += stride) bitmap[i] = 0u;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < npairs; i += stride) first[i] = ~0ull;
}

// bitmap[g][col][b >> 5] |= 1 << (b & 31) for every non-zero (b, col) of group g; first[g][col] = the smallest
// (sample, position) + 1 among them - for a column that a single sample holds that is where its value lies, and
// the update needs no search - or 0 where a sample's row repeats the column (the values then have to be added up)
__global__ __launch_bounds__(256) void k_csr_mark(CsrArgs c, uint32_t *__restrict__ bitmap, unsigned long long *__restrict__ first,
                                                  int words)
{
    const int g = blockIdx.y, b = blockIdx.x;
    const int64_t row = c.row0 + (int64_t)g * c.stride_g + b;
    int64_t p0 = c.rowptr[row], p1 = c.rowptr[row + 1];
    p0 = p0 < 0 ? 0 : p0;
    p1 = p1 > c.nnz ? c.nnz : p1;
    for (int64_t p = p0 + threadIdx.x; p < p1; p += blockDim.x) {
        int32_t col = c.colidx[p];
        if (col < 0 || col >= c.N0) continue;
        const int64_t pair = (int64_t)g * c.N0 + col;
        const uint32_t bit = 1u << (b & 31);
        const uint32_t old = atomicOr(bitmap + pair * words + (b >> 5), bit);
        const bool simple = !(old & bit) && (uint64_t)p < kPosMask;
        atomicMin(first + pair, simple ? (((unsigned long long)b << 40) | (unsigned long long)p) + 1ull : 0ull);
    }
}

// A wavefront takes 64 (group, column) pairs.  For a column that occurs in the batch it finds x[b][col] of the
// samples that hold it (the column's bitmap) and adds x[b][col] * dz[b][:] to its sums in ascending b, one output
// column per lane and pass.  How x[b][col] is found depends on how many of a block of 64 samples hold the column:
// few (most columns occur once or twice in a batch) - the 64 lanes look through a sample's column list together,
// 64 entries per request, one round trip after the row pointers instead of a binary search's chain of dependent
// loads; many (a popular column) - every lane searches its own sample's ascending list, all samples at once.
// Entries of a row that repeat the column are added up in list order either way.
constexpr int kFewSamples = 2;   // (1, 2, 4 measured alike: 180 us per step on the sparse workload; 0 - always the per-lane search - 201, 8: 187)
template <typename D>
__global__ __launch_bounds__(256) void k_csr_update(CsrArgs c, typename D::T *__restrict__ Wt,
                                                    const typename D::T *__restrict__ dz,
                                                    const uint32_t *__restrict__ bitmap,
                                                    const uint64_t *__restrict__ first, int words, float lr)
{
    using T = typename D::T;
    const int lane = threadIdx.x & 63;
    // a wavefront looks at 64 (group, column) pairs at once - most columns do not occur in a batch -
    // and then works through the ones that do, one after the other
    const int64_t w0 = ((int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6)) * 64;
    const int64_t total = (int64_t)c.G * c.N0;
    if (w0 >= total) return;
    int holders = 0;          // samples that hold this lane's column
    uint64_t where = 0;       // and, if it is one, where its value lies
    if (w0 + lane < total) {
        const uint32_t *b0 = bitmap + (w0 + lane) * words;
        for (int i = 0; i < words; ++i) holders += __popc(b0[i]);
        where = first[w0 + lane];
    }
    unsigned long long present = __ballot(holders != 0);
    const T *vals = static_cast<const T *>(c.vals);
    while (present) {
        const int idx = __ffsll((long long)present) - 1;
        const int64_t wid = w0 + idx;
        present &= present - 1;
        const int g = (int)(wid / c.N0);
        const int32_t col = (int32_t)(wid % c.N0);
        const uint32_t *bm = bitmap + wid * words;
        T *wrow = Wt + ((int64_t)g * c.N0 + col) * c.w;
        const T *dzg = dz + (int64_t)g * c.B * c.ld;
        const int n_hold = __shfl(holders, idx);
        const uint64_t wh = ((uint64_t)(uint32_t)__shfl((int)(where >> 32), idx) << 32) | (uint32_t)__shfl((int)(uint32_t)where, idx);
        if (n_hold == 1 && wh != 0ull) {
            // one sample, one entry: value, dz row and old weights in a single round trip
            const int b = (int)((wh - 1) >> 40);
            const float xv = D::up(vals[(wh - 1) & kPosMask]);
            const T *dr = dzg + (int64_t)b * c.ld;
            for (int64_t q = lane; q < c.w; q += 64)
                wrow[q] = D::cvt(D::up(wrow[q]) - lr * (xv * D::ld(dr + q)));
            continue;
        }
        for (int64_t q0 = 0; q0 < c.w; q0 += 256) {          // 4 outputs per lane per pass
            float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            float wold[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {                     // the old weights: asked for now, used at the end
                const int64_t q = q0 + (int64_t)i * 64 + lane;
                wold[i] = q < c.w ? D::up(wrow[q]) : 0.0f;
            }
            for (int b0 = 0; b0 < c.B; b0 += 64) {
                const int b = b0 + lane;
                const bool has = (b < c.B) && ((bm[b >> 5] >> (b & 31)) & 1u);
                unsigned long long m = __ballot(has);
                if (m == 0ull) continue;
                // x[b][col] of the samples that hold the column.  Few of them (the usual case): the 64 lanes look
                // through a sample's column list together, 64 entries per request - one round trip after the row
                // pointers.  Many (a popular column): every lane searches its own sample's ascending list.
                const bool few = __popcll(m) <= kFewSamples;
                float v = 0.0f;
                if (!few && has) {
                    const int64_t row = c.row0 + (int64_t)g * c.stride_g + b;
                    int64_t lo = c.rowptr[row], hi = c.rowptr[row + 1];
                    lo = lo < 0 ? 0 : lo;
                    hi = hi > c.nnz ? c.nnz : hi;
                    const int64_t end = hi;
                    while (lo < hi) {                         // first position with colidx >= col
                        int64_t mid = (lo + hi) >> 1;
                        if (c.colidx[mid] < col) lo = mid + 1; else hi = mid;
                    }
                    // duplicates of a column inside one row are summed
                    for (int64_t p = lo; p < end && c.colidx[p] == col; ++p) v += D::up(vals[p]);
                }
                while (m) {
                    const int src = __ffsll((long long)m) - 1;
                    m &= m - 1;
                    const T *dr = dzg + (int64_t)(b0 + src) * c.ld + q0;
                    float dzv[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {             // the dz row does not depend on the search: asked for first
                        const int64_t q = (int64_t)i * 64 + lane;
                        dzv[i] = q0 + q < c.w ? D::ld(dr + q) : 0.0f;
                    }
                    float xv;
                    if (few) {
                        const int64_t row = c.row0 + (int64_t)g * c.stride_g + b0 + src;
                        int64_t lo = c.rowptr[row], hi = c.rowptr[row + 1];
                        lo = lo < 0 ? 0 : lo;
                        hi = hi > c.nnz ? c.nnz : hi;
                        xv = 0.0f;
                        for (int64_t p0 = lo; p0 < hi; p0 += 64) {
                            const int64_t p = p0 + lane;
                            const bool hit = p < hi && c.colidx[p] == col;
                            const float hv = hit ? D::up(vals[p]) : 0.0f;
                            unsigned long long mh = __ballot(hit);
                            while (mh) {                      // (one entry, unless the row repeats the column)
                                const int sl = __ffsll((long long)mh) - 1;
                                mh &= mh - 1;
                                xv += __shfl(hv, sl);
                            }
                        }
                    } else {
                        xv = __shfl(v, src);
                    }
#pragma unroll
                    for (int i = 0; i < 4; ++i) acc[i] = fmaf(xv, dzv[i], acc[i]);
                }
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int64_t q = q0 + (int64_t)i * 64 + lane;
                if (q < c.w) wrow[q] = D::cvt(wold[i] - lr * acc[i]);
            }
        }
    }
}

hipError_t launch_csr_forward(const CsrArgs &c, const void *Wt, const void *bias, void *h, float *z_out, int dtype,
                              hipStream_t st, bool rowmajor)
{
    int th = c.w >= 256 ? 256 : (c.w > 64 ? 128 : 64);
    dim3 grid((unsigned)((c.w + th - 1) / th), (unsigned)c.B, (unsigned)c.G);
    if (rowmajor) {
        if (dtype == IST_BF16)
            hipLaunchKernelGGL((k_csr_forward<BF16, true>), grid, dim3(th), 0, st, c, (const uint16_t *)Wt,
                               (const uint16_t *)bias, (uint16_t *)h, z_out);
        else
            hipLaunchKernelGGL((k_csr_forward<F32, true>), grid, dim3(th), 0, st, c, (const float *)Wt,
                               (const float *)bias, (float *)h, z_out);
        return hipGetLastError();
    }
    if (dtype == IST_BF16)
        hipLaunchKernelGGL(k_csr_forward<BF16>, grid, dim3(th), 0, st, c, (const uint16_t *)Wt,
                           (const uint16_t *)bias, (uint16_t *)h, z_out);
    else
        hipLaunchKernelGGL(k_csr_forward<F32>, grid, dim3(th), 0, st, c, (const float *)Wt,
                           (const float *)bias, (float *)h, z_out);
    return hipGetLastError();
}

hipError_t launch_csr_update(const CsrArgs &c, void *Wt, const void *dz, uint32_t *bitmap, float lr,
                             int dtype, hipStream_t st)
{
    const int words = (c.B + 31) / 32;
    const int64_t npairs = (int64_t)c.G * c.N0;
    uint64_t *first = reinterpret_cast<uint64_t *>(bitmap + csr_bitmap_words(c.G, c.N0, words));
    hipLaunchKernelGGL(k_csr_clear, dim3(2048), dim3(256), 0, st, bitmap, npairs * words, first, npairs);
    hipLaunchKernelGGL(k_csr_mark, dim3((unsigned)c.B, (unsigned)c.G), dim3(256), 0, st, c, bitmap,
                       reinterpret_cast<unsigned long long *>(first), words);
    const int64_t waves = (npairs + 63) / 64;   // 64 (group, column) pairs per wavefront
    dim3 grid((unsigned)((waves + 3) / 4));
    if (dtype == IST_BF16)
        hipLaunchKernelGGL(k_csr_update<BF16>, grid, dim3(256), 0, st, c, (uint16_t *)Wt,
                           (const uint16_t *)dz, bitmap, first, words, lr);
    else
        hipLaunchKernelGGL(k_csr_update<F32>, grid, dim3(256), 0, st, c, (float *)Wt,
                           (const float *)dz, bitmap, first, words, lr);
    return hipGetLastError();
}

}  // namespace ist
