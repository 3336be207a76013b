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
// Workgroup = 8 wavefronts.  Tiles: all B <= 256 samples x 64 classes (statistics) or 32 classes (backward, where
// four waves make dz of a tile while the other four consume the previous one) x all C <= 128 hidden neurons.
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
__device__ inline int sw4(int r) { return (r >> 2) & 3; }                               //  4 chunks per row (four rows per 256 bytes)
template <int ROWLEN> __device__ inline int tile_off(int r, int e)
{
    static_assert(ROWLEN == 128 || ROWLEN == 64 || ROWLEN == 32, "row lengths in use");
    const int sw = ROWLEN == 128 ? sw16(r) : (ROWLEN == 64 ? sw8(r) : sw4(r));
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

struct SmemStats {
    uint16_t H[kB * kK];         // h_{t-1} of the subnet          [sample][hidden]
    uint16_t W[2][kCT * kK];     // class tiles of W_t              [class][hidden]
    float bias[2][kCT];          // bias of a tile times log2(e); minus infinity past the end of the layer
};

// piece id of a tile of 128-wide rows -> row id / 16, hidden columns 8 (id % 16) .. +7
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

__device__ inline void load_h(uint16_t *H, const WideOutArgs &a, int g)
{
    const uint16_t *h = static_cast<const uint16_t *>(a.h) + (int64_t)g * a.gH;
    const uint16_t *zeros = static_cast<const uint16_t *>(a.zeros);
    constexpr int kPieces = kB * 16 / kThreads;
    uint4 v[kPieces];   // all requests first (none behind a branch), then the stores
#pragma unroll
    for (int i = 0; i < kPieces; ++i) {
        const int id = threadIdx.x + i * kThreads, r = id >> 4, kc = id & 15;
        v[i] = *reinterpret_cast<const uint4 *>(r < a.B && kc * 8 < a.C ? h + (int64_t)r * a.ldh + kc * 8 : zeros);
    }
#pragma unroll
    for (int i = 0; i < kPieces; ++i) store_piece(H, threadIdx.x + i * kThreads, v[i]);
}

// ---------------------------------------------------------------- statistics launch
__global__ __launch_bounds__(kThreads) void k_wide_out_stats(WideOutArgs a)
{
    __shared__ SmemStats sm;
    const int g = blockIdx.x / a.nb, sp = blockIdx.x % a.nb;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint16_t *W = static_cast<const uint16_t *>(a.W) + (int64_t)g * a.gW;
    const uint16_t *bias = a.bias ? static_cast<const uint16_t *>(a.bias) + (int64_t)g * a.gBias : nullptr;
    const int64_t ntiles = (a.N + kCT - 1) / kCT;
    load_h(sm.H, a, g);
    const int s = 32 * wave + (lane & 31), half = lane >> 5;
    const int label = s < a.B ? a.y[(int64_t)g * a.gY + s] : -1;
    float m_run = -INFINITY, s_run = 0.0f;   // running maximum (times log2(e)) and sum of exp(z - maximum)
    const float alpha2 = a.alpha * kLog2e;
    // The pieces of the next tile and its bias are requested while this one is worked on.  No branch around a
    // request and no request that is used where it is issued: one outside the matrices reads a block of zeros, so
    // the wait counters stay exact and the requests stay in flight over the tile's arithmetic.
    const uint16_t *zeros = static_cast<const uint16_t *>(a.zeros);
    auto load_w = [&](int64_t tile, int i) {
        const int id = threadIdx.x + i * kThreads;
        const int64_t r = tile * kCT + (id >> 4);
        const int kc = id & 15;
        const bool ok = tile < ntiles && r < a.N && kc * 8 < a.C;
        return *reinterpret_cast<const uint4 *>(ok ? W + r * a.C + kc * 8 : zeros);
    };
    auto load_b = [&](int64_t tile) {
        const int64_t c = tile * kCT + threadIdx.x;
        const bool ok = threadIdx.x < kCT && bias && tile < ntiles && c < a.N;
        return *(ok ? bias + c : zeros);
    };
    uint4 wreg[2];
    int64_t ti = sp;
#pragma unroll
    for (int i = 0; i < 2; ++i) wreg[i] = load_w(ti, i);
    uint16_t breg = load_b(ti);
    for (int it = 0; ti < ntiles; ti += a.nb, ++it) {
        const int buf = it & 1;
        const int64_t c0 = ti * kCT;
#pragma unroll
        for (int i = 0; i < 2; ++i) store_piece(sm.W[buf], threadIdx.x + i * kThreads, wreg[i]);
        // the bias in units of log2(e), and minus infinity for the classes past the end of the layer: the
        // logits then need one multiply-add each and no test (exp2 of minus infinity is zero)
        if (threadIdx.x < kCT)
            sm.bias[buf][threadIdx.x] = c0 + threadIdx.x < a.N ? bf16_to_f32(breg) * kLog2e : -INFINITY;
#pragma unroll
        for (int i = 0; i < 2; ++i) wreg[i] = load_w(ti + a.nb, i);
        breg = load_b(ti + a.nb);
        __syncthreads();   // (one barrier per tile: the W tiles and the bias alternate between two buffers)
        f32x16 acc[2];
        logits_tile<8>(sm.H, sm.W[buf], wave, lane, acc);
        const bool has_label = label >= c0 && label < c0 + kCT;  // rare: one tile in N / 64 per sample
        float mx = -INFINITY;   // everything below in units of log2(e): z2 = z * log2(e)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int cl = 32 * j + 8 * q + 4 * half;
                const float4 b4 = *reinterpret_cast<const float4 *>(sm.bias[buf] + cl);
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

// ---------------------------------------------------------------- backward launch: two groups of waves
// The exp of the logits is VALU work, the three products that follow are MFMA work, and a SIMD has one pipe of
// each: with all eight waves in the same phase one pipe idles.  Here the waves form two groups of four (one
// wave of each group per SIMD).  Group 0 makes dz: in slot s it computes the logits of class tile s (32 classes,
// all 256 samples), leaves dz in LDS and adds up its share of the bias gradient.  Group 1 consumes the tile one slot
// later: dW and the updated weights.  The workgroup's share of dh stays in registers over all its tiles, 32 samples
// x 128 hidden neurons per wave: a wave of group 0 adds the tile's term for the first 32 of its 64 samples right after
// writing their dz, its partner in group 1 the term for the other 32 one slot later (with all of dh in group 1 that
// group's chain of dependent LDS reads and MFMAs set the pace).  One workgroup barrier per slot; dz and the outgoing
// weights alternate between two buffers, the W tiles between three (tile s is read by group 0, tile s - 1 by
// group 1, tile s + 1 arrives).
constexpr int kC2 = 32;          // classes per tile
constexpr int kDepth = 2;        // W tiles requested ahead (16 bytes per lane each; 3 and 4 measured no faster)

struct SmemBackward {
    uint16_t H[kB * kK];          // h_{t-1} of the subnet          [sample][hidden]
    uint16_t W[3][kC2 * kK];      // class tiles of W_t              [class][hidden]
    uint16_t DZ[2][kB * kC2];     // dz of a tile                    [sample][class]
    uint16_t Wn[2][kC2 * kK];     // updated weights of a tile, on their way out
    float lse2[kB];               // log-sum-exp of the sample times log2(e), plus log2 of the batch size
    int32_t y[kB];
    float bias2[2][kC2];          // bias of a tile times log2(e); minus infinity past the end of the layer
    float braw[4][kC2];           // bias of a tile as stored (tiles s - 2 .. s + 1 are alive in slot s)
    float dbp[4][4][kC2];         // bias gradient of a tile in four partial sums over the samples (tiles s - 2 .. s alive)
};

__global__ __launch_bounds__(kThreads) void k_wide_out_backward(WideOutArgs a)
{
    __shared__ SmemBackward sm;
    const int g = blockIdx.x / a.nb, sp = blockIdx.x % a.nb;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // (uniform: scalar registers)
    const int group = wave >> 2, wg = wave & 3, half = lane >> 5;
    uint16_t *W = static_cast<uint16_t *>(a.W) + (int64_t)g * a.gW;
    uint16_t *bias = a.bias ? static_cast<uint16_t *>(a.bias) + (int64_t)g * a.gBias : nullptr;
    const int64_t ntiles = (a.N + kC2 - 1) / kC2;
    const int nslots = sp < ntiles ? (int)((ntiles - sp + a.nb - 1) / a.nb) : 0;   // tiles sp, sp + nb, ...
    auto tile_c0 = [&](int s) { return ((int64_t)sp + (int64_t)s * a.nb) * kC2; };
    const float alpha2 = a.alpha * kLog2e;

    load_h(sm.H, a, g);
    if (threadIdx.x < kB) {
        const int sx = threadIdx.x;
        sm.lse2[sx] = sx < a.B ? fmaf(a.lse[(int64_t)g * a.B + sx], kLog2e, log2f((float)a.B)) : INFINITY;
        sm.y[sx] = sx < a.B ? a.y[(int64_t)g * a.gY + sx] : -1;
    }
    // the bias of class c0 + threadIdx.x of tile s (threads 0 .. 31), requested ahead like the W pieces: a load that is
    // used in the slot that issues it would make its wave wait for every older request as well
    // (no branch around a request either: one outside the matrices reads a block of zeros, so the wait counters
    // stay exact and requests stay in flight across slots)
    const uint16_t *zeros = static_cast<const uint16_t *>(a.zeros);
    auto load_b = [&](int s) {
        const int64_t c = tile_c0(s) + threadIdx.x;
        const bool ok = threadIdx.x < kC2 && bias && s < nslots && c < a.N;
        return *(ok ? bias + c : zeros);
    };
    auto store_b = [&](int s, uint16_t raw) {   // bias of tile s: in the units of the exponent, and as it is for the update
        if (threadIdx.x < kC2) {
            const float b = bf16_to_f32(raw);
            sm.bias2[s & 1][threadIdx.x] = (s < nslots && tile_c0(s) + threadIdx.x < a.N) ? b * kLog2e : -INFINITY;
            sm.braw[s & 3][threadIdx.x] = b;
        }
    };
    // one 16-byte piece of a W tile per thread: piece id -> class row id / 16, hidden columns 8 (id % 16) .. +7
    auto load_w = [&](int s) {
        const int64_t r = tile_c0(s) + (threadIdx.x >> 4);
        const int kc = threadIdx.x & 15;
        const bool ok = s < nslots && r < a.N && kc * 8 < a.C;
        return *reinterpret_cast<const uint4 *>(ok ? W + r * a.C + kc * 8 : zeros);
    };
    store_piece(sm.W[0], threadIdx.x, load_w(0));
    store_b(0, load_b(0));
    uint4 wreg[kDepth];   // at the top of slot s: the pieces of tiles s + 1 .. s + kDepth, on their way in
    uint16_t breg[kDepth];
#pragma unroll
    for (int j = 0; j < kDepth; ++j) { wreg[j] = load_w(1 + j); breg[j] = load_b(1 + j); }

    // the wave's share of dh: samples 64 wg + 32 group + lane % 32 (the lower half of a wave pair's 64 samples with
    // group 0, which adds to it right after making dz, the upper half with group 1), hidden 32 j + ...
    f32x16 dh[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) dh[j][v] = 0.0f;
    // dh rows += dz (32 samples from row0 on, the tile's 32 classes) x old W of the tile
    auto add_dh = [&](const uint16_t *DZ, const uint16_t *Wt, int row0) {
#pragma unroll
        for (int ks = 0; ks < kC2 / 16; ++ks) {
            const bf16x8 fa = frag_k<kC2>(DZ, row0, ks, lane);            // rows = samples, k = classes
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const bf16x8 fb = frag_m<kK>(Wt, 32 * j, ks, lane);       // rows = hidden,  k = classes
                dh[j] = bf16_mma(fb, fa, dh[j]);
            }
        }
    };
    bf16x8 ones;
#pragma unroll
    for (int i = 0; i < 8; ++i) ones[i] = (__bf16)1.0f;

    // the rows of tile s leave (whole 16-byte pieces) and its bias is updated: b <- b - lr * (four sums, in order)
    auto finish_tile = [&](int s) {
        const int64_t c0 = tile_c0(s);
        const int r = threadIdx.x >> 4, kc = threadIdx.x & 15;
        if (c0 + r < a.N && kc * 8 < a.C)
            *reinterpret_cast<uint4 *>(W + (c0 + r) * a.C + kc * 8) =
                *reinterpret_cast<const uint4 *>(sm.Wn[s & 1] + tile_off<kK>(r, kc * 8));
        if (threadIdx.x < kC2 && bias && c0 + threadIdx.x < a.N) {
            const float(&p)[4][kC2] = sm.dbp[s & 3];
            const float db = ((p[0][threadIdx.x] + p[1][threadIdx.x]) + p[2][threadIdx.x]) + p[3][threadIdx.x];
            bias[c0 + threadIdx.x] = f32_to_bf16(sm.braw[s & 3][threadIdx.x] - a.lr_b * db);
        }
    };
    __syncthreads();   // h, lse, labels, the first W tile and its bias are visible

    // Slot s, both groups: tile s + 1 goes into its LDS buffer (which held tile s - 2), tile s + 1 + kDepth is requested
    // into the registers that this frees, tile s - 2 leaves.  wr / br: the registers of tiles s + 1, s + 1 + kDepth, ...
    auto move_tiles = [&](int s, uint4 &wr, uint16_t &br) {
        store_piece(sm.W[(s + 1) % 3], threadIdx.x, wr);
        store_b(s + 1, br);
        wr = load_w(s + 1 + kDepth);
        br = load_b(s + 1 + kDepth);
        if (s >= 2 && s - 2 < nslots) finish_tile(s - 2);
    };
    // group 0 in slot s: logits of tile s -> dz (bf16) -> LDS; wave wg: samples 64 wg .. 64 wg + 63
    auto produce = [&](int s) {
        if (s < nslots) {
            const uint16_t *Wt = sm.W[s % 3];
            const int64_t c0 = tile_c0(s);
            f32x16 acc[2];
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][v] = 0.0f;
#pragma unroll 4
            for (int ks = 0; ks < kK / 16; ++ks) {
                const bf16x8 fb = frag_k<kK>(Wt, 0, ks, lane);
                const bf16x8 fa0 = frag_k<kK>(sm.H, 64 * wg, ks, lane);
                const bf16x8 fa1 = frag_k<kK>(sm.H, 64 * wg + 32, ks, lane);
                acc[0] = bf16_mma(fb, fa0, acc[0]);
                acc[1] = bf16_mma(fb, fa1, acc[1]);
            }
            // dz = exp2(z2 - lse2 - log2 B) (see k_wide_out_backward: masks through the bias and the
            // log-sum-exp, the label's 1 / B in a branch that few tiles enter)
            uint16_t *DZ = sm.DZ[s & 1];
            const float *b2 = sm.bias2[s & 1];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int row = 64 * wg + 32 * i + (lane & 31);
                const float ls = sm.lse2[row];
                const int label = sm.y[row];
                const bool has_label = label >= c0 && label < c0 + kC2;
                const bool any_label = __builtin_amdgcn_ballot_w64(has_label) != 0ull;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int cl = 8 * q + 4 * half;
                    const float4 b4 = *reinterpret_cast<const float4 *>(b2 + cl);
                    const float bb[4] = {b4.x, b4.y, b4.z, b4.w};
                    float d[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        d[u] = __builtin_amdgcn_exp2f(fmaf(alpha2, acc[i][4 * q + u], bb[u]) - ls);
                    if (any_label) {
#pragma unroll
                        for (int u = 0; u < 4; ++u) d[u] = (c0 + cl + u == label) ? d[u] - a.invB : d[u];
                    }
                    uint2 o;
                    o.x = f32x2_to_bf16x2(d[0], d[1]);
                    o.y = f32x2_to_bf16x2(d[2], d[3]);
                    *reinterpret_cast<uint2 *>(DZ + tile_off<kC2>(row, cl)) = o;
                }
            }
            // the wave's share of the bias gradient: the sum of its 64 samples' dz as stored, per class - a product
            // with a block of ones over the k-steps it has just written (the LDS keeps a wave's accesses in order)
            f32x16 dbv;
#pragma unroll
            for (int v = 0; v < 16; ++v) dbv[v] = 0.0f;
#pragma unroll
            for (int j = 0; j < 4; ++j) dbv = bf16_mma(ones, frag_m<kC2>(DZ, 0, 4 * wg + j, lane), dbv);
            if (half == 0) sm.dbp[s & 3][wg][lane & 31] = dbv[0];
            // and its share of dh, from the 32 rows of dz that this wave wrote first
            add_dh(DZ, Wt, 64 * wg);
        }
    };
    // group 1 in slot s: tile t = s - 1
    auto consume = [&](int t) {
        // ---- dW block of wave wg (32 classes x hidden 32 wg .. +31, k = samples), the updated weights -> LDS ----
        const uint16_t *Wt = sm.W[t % 3];
        const uint16_t *DZ = sm.DZ[t & 1];
        {
            f32x16 dw;
#pragma unroll
            for (int v = 0; v < 16; ++v) dw[v] = 0.0f;
#pragma unroll 4
            for (int ks = 0; ks < kB / 16; ++ks) {
                const bf16x8 fa = frag_m<kC2>(DZ, 0, ks, lane);          // rows = classes, k = samples
                const bf16x8 fb = frag_m<kK>(sm.H, 32 * wg, ks, lane);   // rows = hidden,  k = samples
                dw = bf16_mma(fb, fa, dw);
            }
            const int cl = lane & 31;
            uint16_t *Wn = sm.Wn[t & 1];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int o = tile_off<kK>(cl, 32 * wg + 8 * q + 4 * half);
                const uint2 old = *reinterpret_cast<const uint2 *>(Wt + o);
                const float w0 = __uint_as_float(old.x << 16), w1 = __uint_as_float(old.x & 0xffff0000u);
                const float w2 = __uint_as_float(old.y << 16), w3 = __uint_as_float(old.y & 0xffff0000u);
                uint2 nw;
                nw.x = f32x2_to_bf16x2(w0 - a.lr_w * dw[4 * q], w1 - a.lr_w * dw[4 * q + 1]);
                nw.y = f32x2_to_bf16x2(w2 - a.lr_w * dw[4 * q + 2], w3 - a.lr_w * dw[4 * q + 3]);
                *reinterpret_cast<uint2 *>(Wn + o) = nw;
            }
        }
        // ---- share of dh: the upper 32 of the wave pair's samples (the lower 32 were added by group 0) ----
        add_dh(DZ, Wt, 64 * wg + 32);
    };
    // Slots 0 .. nslots + 1 (the last two only finish tiles), in groups of kDepth so that every slot names its registers.
    // The two groups run loops of their own - what one keeps in registers is not alive in the other - with the same
    // number of workgroup barriers, one at the end of every slot.
    const int nloop = nslots + 2;
    if (group == 0) {
        for (int s0 = 0; s0 < nloop; s0 += kDepth) {
#pragma unroll
            for (int j = 0; j < kDepth; ++j) {
                move_tiles(s0 + j, wreg[j], breg[j]);
                produce(s0 + j);
                __syncthreads();
            }
        }
    } else {
        for (int s0 = 0; s0 < nloop; s0 += kDepth) {
#pragma unroll
            for (int j = 0; j < kDepth; ++j) {
                move_tiles(s0 + j, wreg[j], breg[j]);
                if (s0 + j >= 1 && s0 + j - 1 < nslots) consume(s0 + j - 1);
                __syncthreads();
            }
        }
    }
    const int row = 64 * wg + 32 * group + (lane & 31);
    if (row < a.B) {
        float *out = a.partial + (((int64_t)g * a.nb + sp) * a.B + row) * a.C;
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
    if (!args_ok(a) || !a.pmax || !a.psum || !a.zlabel || !a.zeros) return hipErrorInvalidValue;
    char label[64];
    snprintf(label, sizeof(label), "k_wide_out_stats_bf16_c%d", (int)a.C);
    tag_kernel(label, 2.0 * a.B * (double)a.N * a.C * a.G, (double)a.G * ((double)a.N * a.C + (double)a.B * a.C) * 2.0);
    hipLaunchKernelGGL(k_wide_out_stats, dim3((unsigned)(a.G * a.nb)), dim3(kThreads), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_wide_out_backward(const WideOutArgs &a, hipStream_t st)
{
    if (!args_ok(a) || !a.lse || !a.partial || !a.zeros) return hipErrorInvalidValue;
    char label[64];
    snprintf(label, sizeof(label), "k_wide_out_backward_bf16_c%d", (int)a.C);
    // logits again, dW and dh: three products of 2 B N C flops; W read and written once
    tag_kernel(label, 6.0 * a.B * (double)a.N * a.C * a.G,
               (double)a.G * (2.0 * (double)a.N * a.C * 2.0 + (double)a.B * a.C * 2.0 + (double)a.nb * a.B * a.C * 4.0));
    hipLaunchKernelGGL(k_wide_out_backward, dim3((unsigned)(a.G * a.nb)), dim3(kThreads), 0, st, a);
    return hipGetLastError();
}

}  // namespace ist
