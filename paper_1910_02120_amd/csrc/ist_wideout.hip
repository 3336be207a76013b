// Wide output layer (Section 3.1: the extreme-classification workload, 670,091 classes behind a narrow
// hidden layer), bf16, fused.  For a subnet, the last layer's share of one local SGD step (Section 2.1
// "Training Subnets") is, with h = h_{t-1} [B][C] (C hidden neurons of the subnet) and W = W_t^s [N][C]:
//     z  = alpha h W^T + b                      logits, [B][N]              (never stored: B N floats per subnet)
//     dz = (softmax(z) - onehot(y)) / B          stored rounded to bf16
//     dh = alpha dz W (old W)   dW = dz^T h   db = sum_b dz   W <- W - lr alpha dW   b <- b - lr db
// Two persistent launches do all of it while W is read from HBM twice and written once:
//   statistics: every workgroup keeps h of its subnet in LDS and streams class tiles of W; per sample it keeps
//               a running (max, sum exp) over its tiles and writes one pair at the end, plus the label's logit;
//               (a small kernel merges the pairs into the log-sum-exp and the loss);
//   backward:   same streaming; per class tile the logits are recomputed, dz goes to LDS as bf16 and feeds
//               three more products from there: dW (then the in-place update of the tile's rows, the old
//               weights being the LDS copy), the bias gradient, and this workgroup's share of dh, which stays
//               in registers over all its tiles and is written once as an fp32 partial sum (a finishing kernel
//               adds the workgroups' shares in fixed order and applies the ReLU mask).
// Workgroup = 8 wavefronts.  Tiles: all B <= 256 samples x 64 classes x all C <= 128 hidden neurons.
#include <cstdio>

#include "ist_internal.h"
#include "ist_mfma.h"

namespace ist {

namespace wideout {   // (named: profilers print the kernels as ist::wideout::k_...)

constexpr int kB = 256;          // samples, padded
constexpr int kK = 128;          // hidden neurons of the subnet, padded
constexpr int kCT = 64;          // classes per tile
constexpr int kThreads = 512;
constexpr float kLog2e = 1.4426950408889634f;

// LDS tiles have no row padding.  Every tile is read both ways - as [row][k] with 128-bit reads and as [k][row]
// with the transposing 64-bit reads - and no padding serves both: the first wants a row pitch of 16 bytes times
// an odd number (mod 256), the second 64 or 192 bytes.  Instead the 16-byte chunks of a row are permuted by an
// XOR with a function of the row: 16 consecutive rows put the same chunk into 16 different 16-byte bank slots,
// and 4 consecutive rows put an aligned group of 4 chunks into the 4 different 64-byte bank groups.
__device__ inline int sw16(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }          // 16 chunks per row
__device__ inline int sw8(int r) { return (((r >> 1) & 1) << 2) | ((r >> 2) & 3); }   //  8 chunks per row (two rows per 256 bytes)
template <int ROWLEN> __device__ inline int tile_off(int r, int e)
{
    static_assert(ROWLEN == 128 || ROWLEN == 64, "row lengths in use");
    const int sw = ROWLEN == 128 ? sw16(r) : sw8(r);
    return r * ROWLEN + ((((e >> 3) ^ sw) << 3) | (e & 7));
}
// fragments of a swizzled tile: rows rb .. rb + 31, k-step ks, for a tile kept [row][k] / [k][row]
template <int ROWLEN> __device__ inline bf16x8 frag_k(const uint16_t *t, int rb, int ks, int lane)
{
    return *reinterpret_cast<const bf16x8 *>(t + tile_off<ROWLEN>(rb + (lane & 31), ks * 16 + (lane >> 5) * 8));
}
template <int ROWLEN> __device__ inline bf16x8 frag_m(const uint16_t *t, int rb, int ks, int lane)
{
    const int q = lane & 15;
    const int m = rb + ((lane >> 4) & 1) * 16 + 4 * (q & 3);
    const int k = ks * 16 + (lane >> 5) * 8 + (q >> 2);
    typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(t + tile_off<ROWLEN>(k, m)));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(t + tile_off<ROWLEN>(k + 4, m)));
    s16x8 r = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, r);
}

struct Smem {
    uint16_t H[kB * kK];         // h_{t-1} of the subnet          [sample][hidden]
    uint16_t W[2][kCT * kK];     // class tiles of W_t              [class][hidden]
    uint16_t DZ[kB * kCT];       // dz of the tile                  [sample][class]
    uint16_t Wn[kCT * kK];       // updated weights of the tile, on their way out
    float lse2[kB];              // log-sum-exp of the sample times log2(e), plus log2 of the batch size
    int32_t y[kB];
    float bias[kCT];
    float dbp[4][kCT];           // bias gradient of the tile in four partial sums over the samples
};

// 16-byte pieces of a [rows][C] bf16 matrix with row pitch `ld`: piece id -> row id / 16, hidden columns
// 8 (id % 16) .. +7; rows >= rows_ok and columns >= C read as zero.
__device__ inline uint4 load_piece(const uint16_t *src, int64_t ld, int id, int64_t row0, int64_t rows_ok, int C)
{
    const int r = id >> 4, kc = id & 15;
    const bool ok = row0 + r < rows_ok && kc * 8 < C;
    return ok ? *reinterpret_cast<const uint4 *>(src + (row0 + r) * ld + kc * 8) : uint4{0, 0, 0, 0};
}
__device__ inline void store_piece(uint16_t *tile, int id, uint4 v)
{
    *reinterpret_cast<uint4 *>(tile + tile_off<kK>(id >> 4, (id & 15) * 8)) = v;
}

// logits of the wave's 32 samples against the 64 classes of a W tile:
// acc[j][4 q + u] = sum_k h[32 wave + lane % 32][k] W[32 j + 8 q + 4 (lane / 32) + u][k]
template <int UNROLL>
__device__ inline void logits_tile(const uint16_t *Hs, const uint16_t *Wt, int wave, int lane, f32x16 (&acc)[2])
{
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.0f;
#pragma unroll UNROLL
    for (int ks = 0; ks < kK / 16; ++ks) {
        const bf16x8 fa = frag_k<kK>(Hs, 32 * wave, ks, lane);
        const bf16x8 fb0 = frag_k<kK>(Wt, 0, ks, lane);
        const bf16x8 fb1 = frag_k<kK>(Wt, 32, ks, lane);
        acc[0] = bf16_mma(fb0, fa, acc[0]);
        acc[1] = bf16_mma(fb1, fa, acc[1]);
    }
}

__device__ inline void load_h(Smem &sm, const WideOutArgs &a, int g)
{
    const uint16_t *h = static_cast<const uint16_t *>(a.h) + (int64_t)g * a.gH;
#pragma unroll
    for (int i = 0; i < kB * 16 / kThreads; ++i) {
        const int id = threadIdx.x + i * kThreads;
        store_piece(sm.H, id, load_piece(h, a.ldh, id, 0, a.B, a.C));
    }
}

// ---------------------------------------------------------------- statistics launch
__global__ __launch_bounds__(kThreads) void k_wide_out_stats(WideOutArgs a)
{
    __shared__ Smem sm;
    const int g = blockIdx.x / a.nb, sp = blockIdx.x % a.nb;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint16_t *W = static_cast<const uint16_t *>(a.W) + (int64_t)g * a.gW;
    const uint16_t *bias = a.bias ? static_cast<const uint16_t *>(a.bias) + (int64_t)g * a.gBias : nullptr;
    const int64_t ntiles = (a.N + kCT - 1) / kCT;
    load_h(sm, a, g);
    const int s = 32 * wave + (lane & 31), half = lane >> 5;
    const int label = s < a.B ? a.y[(int64_t)g * a.gY + s] : -1;
    float m_run = -INFINITY, s_run = 0.0f;   // running maximum (times log2(e)) and sum of exp(z - maximum)
    const float alpha2 = a.alpha * kLog2e;
    uint4 wreg[2];
    int64_t ti = sp;
#pragma unroll
    for (int i = 0; i < 2; ++i) wreg[i] = load_piece(W, a.C, threadIdx.x + i * kThreads, ti * kCT, a.N, a.C);
    for (int it = 0; ti < ntiles; ti += a.nb, ++it) {
        const int buf = it & 1;
        const int64_t c0 = ti * kCT;
#pragma unroll
        for (int i = 0; i < 2; ++i) store_piece(sm.W[buf], threadIdx.x + i * kThreads, wreg[i]);
        // the bias in units of log2(e), and minus infinity for the classes past the end of the layer: the
        // logits then need one multiply-add each and no test (exp2 of minus infinity is zero)
        if (threadIdx.x < kCT)
            sm.bias[threadIdx.x] = c0 + threadIdx.x < a.N ? (bias ? bf16_to_f32(bias[c0 + threadIdx.x]) * kLog2e : 0.0f) : -INFINITY;
#pragma unroll
        for (int i = 0; i < 2; ++i)   // the next tile's pieces fly during this tile's arithmetic
            wreg[i] = load_piece(W, a.C, threadIdx.x + i * kThreads, (ti + a.nb) * kCT, a.N, a.C);
        __syncthreads();
        f32x16 acc[2];
        logits_tile<8>(sm.H, sm.W[buf], wave, lane, acc);
        const bool has_label = label >= c0 && label < c0 + kCT;  // rare: one tile in N / 64 per sample
        float mx = -INFINITY;   // everything below in units of log2(e): z2 = z * log2(e)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int cl = 32 * j + 8 * q + 4 * half;
                const float4 b4 = *reinterpret_cast<const float4 *>(sm.bias + cl);
                const float bb[4] = {b4.x, b4.y, b4.z, b4.w};
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const float z2 = fmaf(alpha2, acc[j][4 * q + u], bb[u]);
                    acc[j][4 * q + u] = z2;
                    mx = fmaxf(mx, z2);
                }
            }
        if (__builtin_amdgcn_ballot_w64(has_label) != 0ull) {
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    if (c0 + 32 * j + 8 * (v >> 2) + 4 * half + (v & 3) == label)
                        a.zlabel[(int64_t)g * a.B + s] = acc[j][v] * (1.0f / kLog2e);
        }
        if (mx > -INFINITY) {
            const float m_new = fmaxf(m_run, mx);
            float se = 0.0f;
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) se += __builtin_amdgcn_exp2f(acc[j][v] - m_new);
            s_run = s_run * __builtin_amdgcn_exp2f(m_run - m_new) + se;
            m_run = m_new;
        }
        __syncthreads();   // the bias is free again (the W tiles alternate between two buffers)
    }
    // the two halves of a row (lane, lane ^ 32), then one pair per sample and workgroup
    const float m_o = __shfl_xor(m_run, 32), s_o = __shfl_xor(s_run, 32);
    const float m_all = fmaxf(m_run, m_o);
    float s_all = 0.0f;
    if (m_all > -INFINITY)
        s_all = (m_run > -INFINITY ? s_run * __builtin_amdgcn_exp2f(m_run - m_all) : 0.0f) +
                (m_o > -INFINITY ? s_o * __builtin_amdgcn_exp2f(m_o - m_all) : 0.0f);
    if (half == 0 && s < a.B) {
        const int64_t pi = ((int64_t)g * a.nb + sp) * a.B + s;
        a.pmax[pi] = m_all * (1.0f / kLog2e);   // back to natural units for the merge
        a.psum[pi] = s_all;
    }
}

// ---------------------------------------------------------------- backward launch
__global__ __launch_bounds__(kThreads) void k_wide_out_backward(WideOutArgs a)
{
    __shared__ Smem sm;
    const int g = blockIdx.x / a.nb, sp = blockIdx.x % a.nb;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint16_t *W = static_cast<uint16_t *>(a.W) + (int64_t)g * a.gW;
    uint16_t *bias = a.bias ? static_cast<uint16_t *>(a.bias) + (int64_t)g * a.gBias : nullptr;
    const int64_t ntiles = (a.N + kCT - 1) / kCT;
    load_h(sm, a, g);
    if (threadIdx.x < kB) {
        const int sx = threadIdx.x;
        sm.lse2[sx] = sx < a.B ? fmaf(a.lse[(int64_t)g * a.B + sx], kLog2e, log2f((float)a.B)) : INFINITY;
        sm.y[sx] = sx < a.B ? a.y[(int64_t)g * a.gY + sx] : -1;
    }
    const int s = 32 * wave + (lane & 31), half = lane >> 5;
    f32x16 dh[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) dh[j][v] = 0.0f;
    bf16x8 ones;
#pragma unroll
    for (int i = 0; i < 8; ++i) ones[i] = (__bf16)1.0f;
    const float alpha2 = a.alpha * kLog2e;

    // bias of the class this thread looks after (threads 0 .. 63), as loaded for the tile in progress
    float b_old = 0.0f;
    int64_t b_class = -1, prev_c0 = -1;
    auto finish_tile = [&]() {
        // b <- b - lr * (the four partial sums, in order); the updated rows of W_t leave as whole 16-byte pieces
        if (threadIdx.x < kCT && bias && b_class >= 0 && b_class < a.N) {
            const float db = ((sm.dbp[0][threadIdx.x] + sm.dbp[1][threadIdx.x]) + sm.dbp[2][threadIdx.x]) + sm.dbp[3][threadIdx.x];
            bias[b_class] = f32_to_bf16(b_old - a.lr_b * db);
        }
        if (prev_c0 >= 0) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int id = threadIdx.x + i * kThreads, r = id >> 4, kc = id & 15;
                if (prev_c0 + r < a.N && kc * 8 < a.C)
                    *reinterpret_cast<uint4 *>(W + (prev_c0 + r) * a.C + kc * 8) =
                        *reinterpret_cast<const uint4 *>(sm.Wn + tile_off<kK>(r, kc * 8));
            }
        }
    };

    uint4 wreg[2];
    int64_t ti = sp;
#pragma unroll
    for (int i = 0; i < 2; ++i) wreg[i] = load_piece(W, a.C, threadIdx.x + i * kThreads, ti * kCT, a.N, a.C);
    if (ti < ntiles) {
#pragma unroll
        for (int i = 0; i < 2; ++i) store_piece(sm.W[0], threadIdx.x + i * kThreads, wreg[i]);
    }
    for (int it = 0; ti < ntiles; ti += a.nb, ++it) {
        const int buf = it & 1;
        const int64_t c0 = ti * kCT;
        const uint16_t *Wt = sm.W[buf];
#pragma unroll
        for (int i = 0; i < 2; ++i)   // the next tile's pieces fly during this tile's arithmetic
            wreg[i] = load_piece(W, a.C, threadIdx.x + i * kThreads, (ti + a.nb) * kCT, a.N, a.C);
        finish_tile();                // of the tile before (complete since the barrier that ended it)
        prev_c0 = c0;
        if (threadIdx.x < kCT) {
            b_class = c0 + threadIdx.x;
            b_old = (bias && b_class < a.N) ? bf16_to_f32(bias[b_class]) : 0.0f;
            sm.bias[threadIdx.x] = b_class < a.N ? b_old * kLog2e : -INFINITY;
        }
        __syncthreads();   // B1: bias (and, the first time, h, lse, labels and the first W tile) visible
        // ---- logits -> dz (bf16) -> LDS ----
        {
            f32x16 acc[2];
            logits_tile<2>(sm.H, Wt, wave, lane, acc);
            // dz = exp2(z2 - lse2 - log2 B) with z2 = alpha2 acc + bias2 in units of log2(e); classes past the end
            // of the layer carry a bias of minus infinity and samples past the batch a log-sum-exp of plus
            // infinity, so they come out as exact zeros without a test; the label's 1 / B is taken off in a
            // branch that few tiles enter (a sample's label lies in one tile of N / 64)
            const float ls = sm.lse2[s];
            const int label = sm.y[s];
            const bool has_label = label >= c0 && label < c0 + kCT;
            const bool any_label = __builtin_amdgcn_ballot_w64(has_label) != 0ull;
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int cl = 32 * j + 8 * q + 4 * half;
                    const float4 b4 = *reinterpret_cast<const float4 *>(sm.bias + cl);
                    const float bb[4] = {b4.x, b4.y, b4.z, b4.w};
                    float d[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        d[u] = __builtin_amdgcn_exp2f(fmaf(alpha2, acc[j][4 * q + u], bb[u]) - ls);
                    if (any_label) {
#pragma unroll
                        for (int u = 0; u < 4; ++u) d[u] = (c0 + cl + u == label) ? d[u] - a.invB : d[u];
                    }
                    uint2 o;
                    o.x = f32x2_to_bf16x2(d[0], d[1]);
                    o.y = f32x2_to_bf16x2(d[2], d[3]);
                    *reinterpret_cast<uint2 *>(sm.DZ + tile_off<kCT>(s, cl)) = o;
                }
        }
        // the next W tile into the other buffer (last read before the barrier that ended the tile before)
#pragma unroll
        for (int i = 0; i < 2; ++i) store_piece(sm.W[buf ^ 1], threadIdx.x + i * kThreads, wreg[i]);
        __syncthreads();   // B2: dz tile complete
        // ---- dW block (32 classes x 32 hidden per wave, k = samples), the bias gradient of those classes
        //      (a product with a block of ones, every fourth k-step per wave), the updated weights -> LDS ----
        {
            const int ci = wave >> 2, hj = wave & 3;
            f32x16 dw, dbv;
#pragma unroll
            for (int v = 0; v < 16; ++v) { dw[v] = 0.0f; dbv[v] = 0.0f; }
#pragma unroll 4
            for (int ks = 0; ks < kB / 16; ++ks) {
                const bf16x8 fa = frag_m<kCT>(sm.DZ, 32 * ci, ks, lane);   // rows = classes, k = samples
                const bf16x8 fb = frag_m<kK>(sm.H, 32 * hj, ks, lane);     // rows = hidden,  k = samples
                dw = bf16_mma(fb, fa, dw);
                if ((ks & 3) == hj) dbv = bf16_mma(ones, fa, dbv);
            }
            const int cl = 32 * ci + (lane & 31);
            if (half == 0) sm.dbp[hj][cl] = dbv[0];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int jj = 32 * hj + 8 * q + 4 * half;
                const int o = tile_off<kK>(cl, jj);
                const uint2 old = *reinterpret_cast<const uint2 *>(Wt + o);
                const float w0 = __uint_as_float(old.x << 16), w1 = __uint_as_float(old.x & 0xffff0000u);
                const float w2 = __uint_as_float(old.y << 16), w3 = __uint_as_float(old.y & 0xffff0000u);
                uint2 nw;
                nw.x = f32x2_to_bf16x2(w0 - a.lr_w * dw[4 * q], w1 - a.lr_w * dw[4 * q + 1]);
                nw.y = f32x2_to_bf16x2(w2 - a.lr_w * dw[4 * q + 2], w3 - a.lr_w * dw[4 * q + 3]);
                *reinterpret_cast<uint2 *>(sm.Wn + o) = nw;
            }
        }
        // ---- this workgroup's share of dh: 32 samples x 128 hidden per wave, k = the tile's classes, old W ----
#pragma unroll 2
        for (int ks = 0; ks < kCT / 16; ++ks) {
            const bf16x8 fa = frag_k<kCT>(sm.DZ, 32 * wave, ks, lane);       // rows = samples, k = classes
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const bf16x8 fb = frag_m<kK>(Wt, 32 * j, ks, lane);          // rows = hidden,  k = classes
                dh[j] = bf16_mma(fb, fa, dh[j]);
            }
        }
        __syncthreads();   // B3: everybody is done with the dz tile and this W tile; Wn and the partial sums are written
    }
    finish_tile();
    if (s < a.B) {
        float *out = a.partial + (((int64_t)g * a.nb + sp) * a.B + s) * a.C;
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int jj = 32 * j + 8 * q + 4 * half;
                if (jj < a.C)
                    *reinterpret_cast<float4 *>(out + jj) =
                        make_float4(dh[j][4 * q], dh[j][4 * q + 1], dh[j][4 * q + 2], dh[j][4 * q + 3]);
            }
    }
}

bool args_ok(const WideOutArgs &a)
{
    return a.G > 0 && a.B > 0 && a.B <= kB && a.C > 0 && a.C <= kK && a.C % 8 == 0 && a.N > 0 && a.nb > 0 &&
           reinterpret_cast<uintptr_t>(a.h) % 16 == 0 && a.ldh % 8 == 0 && a.gH % 8 == 0 &&
           reinterpret_cast<uintptr_t>(a.W) % 16 == 0 && a.gW % 8 == 0;
}

}  // namespace wideout
using namespace wideout;

bool wide_out_supported(int dtype, int32_t B, int64_t C, int64_t N)
{
    return dtype == IST_BF16 && B >= 1 && B <= kB && C >= 8 && C <= kK && C % 8 == 0 && N > 4096;
}

// 256 compute units, one resident workgroup each (the shared memory of a workgroup fills a unit)
int wide_out_workgroups(int32_t G)
{
    const int n = 256 / (G > 0 ? G : 1);
    return n < 1 ? 1 : (n > 64 ? 64 : n);
}

hipError_t launch_wide_out_stats(const WideOutArgs &a, hipStream_t st)
{
    if (!args_ok(a) || !a.pmax || !a.psum || !a.zlabel) return hipErrorInvalidValue;
    char label[64];
    snprintf(label, sizeof(label), "k_wide_out_stats_bf16_c%d", (int)a.C);
    tag_kernel(label, 2.0 * a.B * (double)a.N * a.C * a.G, (double)a.G * ((double)a.N * a.C + (double)a.B * a.C) * 2.0);
    hipLaunchKernelGGL(k_wide_out_stats, dim3((unsigned)(a.G * a.nb)), dim3(kThreads), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_wide_out_backward(const WideOutArgs &a, hipStream_t st)
{
    if (!args_ok(a) || !a.lse || !a.partial) return hipErrorInvalidValue;
    char label[64];
    snprintf(label, sizeof(label), "k_wide_out_backward_bf16_c%d", (int)a.C);
    // logits again, dW and dh: three products of 2 B N C flops; W read and written once
    tag_kernel(label, 6.0 * a.B * (double)a.N * a.C * a.G,
               (double)a.G * (2.0 * (double)a.N * a.C * 2.0 + (double)a.B * a.C * 2.0 + (double)a.nb * a.B * a.C * 4.0));
    hipLaunchKernelGGL(k_wide_out_backward, dim3((unsigned)(a.G * a.nb)), dim3(kThreads), 0, st, a);
    return hipGetLastError();
}

}  // namespace ist
