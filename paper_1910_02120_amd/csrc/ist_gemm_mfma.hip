// MFMA grouped GEMM for the subnet SGD step (gfx950).
//
//   C_g[m][n] = sum_k A_g(m,k) * B_g(n,k),   g = subnet (part of the 1-D tile index)
//
// Each operand is either K-contiguous (rows of k values) or M-contiguous (the
// matrix is stored with k as the slow index).  The three products of a layer
// (Section 2.1 "Training Subnets": forward, back-propagation, SGD update) are
//   forward         A = h_{l-1} (K-contig)   B = W_l (K-contig)
//   backward data   A = dz_l    (K-contig)   B = W_l (M-contig: k runs over rows of W_l)
//   backward weight A = dz_l    (M-contig)   B = h_{l-1} (M-contig)
// so no operand is ever stored twice or transposed in memory.  A wide output layer keeps its
// dz transposed (classes x samples, written by the second cross-entropy pass); there the
// backward-data product reads A M-contiguous and the update reads it K-contiguous.
//
// bf16: v_mfma_f32_32x32x16_bf16.  K-contiguous tiles sit in LDS as [row][k] and a
// lane's 8 consecutive k values are one 128-bit LDS read; M-contiguous tiles sit as
// [k][row] exactly as in memory and the fragment is produced by the transposing LDS
// read ds_read_b64_tr_b16 (two per fragment).
// f32: v_mfma_f32_32x32x2_f32, one value per lane and operand; both LDS layouts
// are read with plain 32-bit loads.
//
// Workgroup = 4*KG wavefronts: a 2x2 arrangement over the BM x BN tile, times KG
// "k-groups" that share the LDS tiles and each take every KG-th MFMA k-step (their
// accumulators are added through LDS in fixed order at the end).  Small problems use
// 64x64 tiles with KG > 1 so that all SIMDs have a wave; large ones 128x128, KG = 1.
// Global loads are 16 bytes per lane and run ST k-tiles ahead in registers.
// The epilogue goes through LDS so that every lane owns 8 consecutive columns of a
// row: bias/ReLU, the ReLU mask, or the in-place SGD update then use 16-byte accesses
// (the row statistics of a wide output layer are taken from the accumulators directly).
// The update products of several small layers, and their bias updates, can share one launch.
#include "ist_internal.h"
#include "ist_bias_block.h"
#include "ist_mfma.h"

#include <cmath>
#include <cstdio>

namespace ist {

template <typename D, int KT> struct Mma;   // KT: k extent of one LDS tile

template <int KT> struct Mma<BF16, KT> {
    using E = uint16_t;
    using Frag = bf16x8;
    static constexpr int CH = 8;          // elements per 16-byte chunk
    static constexpr int KSTEPS = KT / 16;
    static constexpr int ld_k(int) { return KT + 8; }          // [row][k] row pitch (elements)
    // [k][row] row pitch: +32 elements (16 words) keeps the four k-rows one transposing
    // read touches in distinct bank groups (measured: SQ_LDS_BANK_CONFLICT drops ~10x vs +16)
    static constexpr int ld_m(int rows) { return rows + 32; }
    __device__ static inline f32x16 mma(Frag a, Frag b, f32x16 c) { return bf16_mma(a, b, c); }
    __device__ static inline void store_k(E *lds, int row, int kc, uint4 v, int ld)
    {
        *reinterpret_cast<uint4 *>(lds + row * ld + kc * CH) = v;
    }
    __device__ static inline Frag frag_k(const E *lds, int rb, int ks, int lane, int ld) { return bf16_frag_k(lds, rb, ks, lane, ld); }
    __device__ static inline Frag frag_m(const E *lds, int rb, int ks, int lane, int ld) { return bf16_frag_m(lds, rb, ks, lane, ld); }
};

template <int KT> struct Mma<F32, KT> {
    using E = float;
    using Frag = float;
    static constexpr int CH = 4;
    static constexpr int KSTEPS = KT / 2;
    static constexpr int ld_k(int) { return KT + 1; }
    static constexpr int ld_m(int rows) { return rows + 4; }
    __device__ static inline f32x16 mma(Frag a, Frag b, f32x16 c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
    }
    __device__ static inline void store_k(E *lds, int row, int kc, uint4 v, int ld)
    {
        E *p = lds + row * ld + kc * CH;
        p[0] = __uint_as_float(v.x); p[1] = __uint_as_float(v.y);
        p[2] = __uint_as_float(v.z); p[3] = __uint_as_float(v.w);
    }
    __device__ static inline Frag frag_k(const E *lds, int rb, int ks, int lane, int ld)
    {
        return lds[(rb + (lane & 31)) * ld + ks * 2 + (lane >> 5)];
    }
    __device__ static inline Frag frag_m(const E *lds, int rb, int ks, int lane, int ld)
    {
        return lds[(ks * 2 + (lane >> 5)) * ld + rb + (lane & 31)];
    }
};

// One operand tile: ROWS rows (m or n) by KT k values, loaded by NT threads.
template <typename D, bool KCONTIG, int ROWS, int NT, int KT>
struct Tile {
    using M = Mma<D, KT>;
    using E = typename M::E;
    static constexpr int CH = M::CH;
    static constexpr int LD = KCONTIG ? M::ld_k(ROWS) : M::ld_m(ROWS);
    static constexpr int ELEMS = KCONTIG ? ROWS * LD : KT * LD;
    static constexpr int CHUNKS = ROWS * KT / CH;
    static constexpr int PER = (CHUNKS + NT - 1) / NT;   // chunks per thread

    struct Regs { uint4 v[PER]; };

    // chunk c -> (row, k) of its first element inside the tile
    __device__ static inline void coords(int c, int &row, int &k)
    {
        if (KCONTIG) { row = c / (KT / CH); k = (c % (KT / CH)) * CH; }
        else         { k = c / (ROWS / CH); row = (c % (ROWS / CH)) * CH; }
    }

    // s_row / s_k: element strides of the row index and of k (one of them is 1).
    // VEC: one unconditional 16-byte load per chunk; a chunk outside the operand is
    // read from a block of zeros instead, so nothing branches around the loads, nothing
    // has to touch the loaded registers before they are stored to LDS, and the loads
    // stay in flight across k-tiles.
    template <bool VEC>
    __device__ static inline void load(Regs &r, const E *base, const E *zeros, int64_t s_row, int64_t s_k,
                                       int row0, int rows_total, int k0, int K)
    {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int c = threadIdx.x + i * NT;
            int row, k;
            coords(c, row, k);
            const int gr = row0 + row, gk = k0 + k;
            const bool ok = (CHUNKS % NT == 0 || c < CHUNKS) && gr < rows_total && gk < K;
            const E *p = ok ? base + ((int64_t)gr * s_row + (int64_t)gk * s_k) : zeros;
            uint4 v;
            if (VEC) {
                v = *reinterpret_cast<const uint4 *>(p);
            } else {
                E tmp[CH];
#pragma unroll
                for (int e = 0; e < CH; ++e) {
                    const bool oke = ok && (KCONTIG ? (gk + e < K) : (gr + e < rows_total));
                    tmp[e] = (oke ? p : zeros)[oke ? e : 0];
                }
                __builtin_memcpy(&v, tmp, 16);
            }
            r.v[i] = v;
        }
    }

    __device__ static inline void store(E *lds, const Regs &r)
    {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int c = threadIdx.x + i * NT;
            if (CHUNKS % NT == 0 || c < CHUNKS) {
                int row, k;
                coords(c, row, k);
                if (KCONTIG) M::store_k(lds, row, k / CH, r.v[i], LD);
                else *reinterpret_cast<uint4 *>(lds + k * LD + row) = r.v[i];
            }
        }
    }

    __device__ static inline typename M::Frag frag(const E *lds, int rb, int ks, int lane)
    {
        return KCONTIG ? M::frag_k(lds, rb, ks, lane, LD) : M::frag_m(lds, rb, ks, lane, LD);
    }
};

// ---------------------------------------------------------------- 8-wide row accesses
template <typename T> struct Row8;
template <> struct Row8<uint16_t> {
    __device__ static inline void ld(const uint16_t *p, bool vec, int nv, float (&o)[8])
    {
        if (vec) {
            uint4 r = *reinterpret_cast<const uint4 *>(p);
            const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                o[2 * i] = __uint_as_float(w[i] << 16);
                o[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) o[i] = i < nv ? bf16_to_f32(p[i]) : 0.0f;
        }
    }
    __device__ static inline void st(uint16_t *p, bool vec, int nv, const float (&v)[8])
    {
        if (vec) {
            uint32_t w[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                w[i] = f32x2_to_bf16x2(v[2 * i], v[2 * i + 1]);
            *reinterpret_cast<uint4 *>(p) = make_uint4(w[0], w[1], w[2], w[3]);
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (i < nv) p[i] = f32_to_bf16(v[i]);
        }
    }
};
template <> struct Row8<float> {
    __device__ static inline void ld(const float *p, bool vec, int nv, float (&o)[8])
    {
        if (vec) {
            float4 a = *reinterpret_cast<const float4 *>(p);
            float4 b = *reinterpret_cast<const float4 *>(p + 4);
            o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w; o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) o[i] = i < nv ? p[i] : 0.0f;
        }
    }
    __device__ static inline void st(float *p, bool vec, int nv, const float (&v)[8])
    {
        if (vec) {
            *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
            *reinterpret_cast<float4 *>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (i < nv) p[i] = v[i];
        }
    }
};

// The 8 storage-type values an epilogue combines with its 8 results (the old weights for the
// update, the activations for the ReLU mask), fetched ahead of time as raw 16-byte pieces.
template <typename T> struct Pre8 { uint4 v[sizeof(T) / 2]; };
template <typename T> __device__ inline void pre8_decode(const Pre8<T> &r, float (&o)[8]);
template <> __device__ inline void pre8_decode<uint16_t>(const Pre8<uint16_t> &r, float (&o)[8])
{
    const uint32_t w[4] = {r.v[0].x, r.v[0].y, r.v[0].z, r.v[0].w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        o[2 * i] = __uint_as_float(w[i] << 16);
        o[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
}
template <> __device__ inline void pre8_decode<float>(const Pre8<float> &r, float (&o)[8])
{
    o[0] = __uint_as_float(r.v[0].x); o[1] = __uint_as_float(r.v[0].y);
    o[2] = __uint_as_float(r.v[0].z); o[3] = __uint_as_float(r.v[0].w);
    o[4] = __uint_as_float(r.v[1].x); o[5] = __uint_as_float(r.v[1].y);
    o[6] = __uint_as_float(r.v[1].z); o[7] = __uint_as_float(r.v[1].w);
}

// Epilogue for 8 consecutive columns n0..n0+7 of row m (gz: output group index).
// pre: values fetched ahead for this chunk (HASPRE; used on the 16-byte path only).
// bias8: the bias of these 8 columns (zeros without bias), fetched once per tile by the caller.
template <typename D, int EPI, bool HASPRE = false>
__device__ inline void epi8(const GemmArgs &a, int g, int gz, int m, int n0, float (&val)[8], bool vecC,
                            const float (&bias8)[8], const Pre8<typename D::T> &pre = Pre8<typename D::T>{})
{
    using T = typename D::T;
    if (m >= a.M || n0 >= a.N) return;
    const int nv = a.N - n0 < 8 ? a.N - n0 : 8;
    const bool vec = vecC && nv == 8;
    const int64_t ci = (int64_t)gz * a.gC + (int64_t)m * a.ldc + n0;
    if (EPI == EPI_PARTIAL) {
        Row8<float>::st(static_cast<float *>(a.C) + ci, vec, nv, val);
        return;
    }
    if (EPI == EPI_FWD_RELU || EPI == EPI_FWD_LOGITS) {
#pragma unroll
        for (int i = 0; i < 8; ++i) val[i] = fmaf(a.alpha, val[i], bias8[i]);   // alpha = 1: exactly val + bias
        if (EPI == EPI_FWD_RELU) {
#pragma unroll
            for (int i = 0; i < 8; ++i) val[i] = val[i] > 0.0f ? val[i] : 0.0f;
            Row8<T>::st(static_cast<T *>(a.C) + ci, vec, nv, val);
        } else {
            Row8<float>::st(static_cast<float *>(a.C) + ci, vec, nv, val);
        }
        return;
    }
    float o[8];
    if (EPI == EPI_BWD_DATA) {
        if (HASPRE && vec) pre8_decode<T>(pre, o);
        else Row8<T>::ld(static_cast<const T *>(a.mask) + (int64_t)g * a.gMask + (int64_t)m * a.ldm + n0, vec, nv, o);
#pragma unroll
        for (int i = 0; i < 8; ++i) val[i] = o[i] > 0.0f ? a.alpha * val[i] : 0.0f;
    } else {   // EPI_UPDATE
        if (HASPRE && vec) pre8_decode<T>(pre, o);
        else Row8<T>::ld(static_cast<const T *>(a.C) + ci, vec, nv, o);
#pragma unroll
        for (int i = 0; i < 8; ++i) val[i] = o[i] - a.lr * val[i];
    }
    Row8<T>::st(static_cast<T *>(a.C) + ci, vec, nv, val);
}


// EPI_DZT: rows are classes, columns samples: dz^T[m][n] = (exp(z - lse_n) - [m == y_n]) / B in the storage
// dtype.  ls8: the samples' log-sum-exp times log2(e), lab8 their labels, brow the bias of class m.
// Returns the sum of the values as stored (the chunk's share of the bias gradient of class m).
template <typename D>
__device__ inline float epi_dzt(const GemmArgs &a, int g, int m, int n0, float (&val)[8], bool vecC, float brow,
                                const int (&lab8)[8], const float (&ls8)[8])
{
    using T = typename D::T;
    if (m >= a.M || n0 >= a.N) return 0.0f;
    const int nv = a.N - n0 < 8 ? a.N - n0 : 8;
    const bool vec = vecC && nv == 8;
    constexpr float kLog2e = 1.4426950408889634f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const float z = fmaf(a.alpha, val[i], brow);
        val[i] = __builtin_amdgcn_exp2f(fmaf(z, kLog2e, -ls8[i])) * a.invB;
        val[i] = lab8[i] == m ? val[i] - a.invB : val[i];
    }
    Row8<T>::st(static_cast<T *>(a.C) + (int64_t)g * a.gC + (int64_t)m * a.ldc + n0, vec, nv, val);
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) s += i < nv ? D::up(D::cvt(val[i])) : 0.0f;
    return s;
}

template <int A, int B> struct MaxOf { static constexpr int v = A > B ? A : B; };

// splits > 1 (EPI_PARTIAL only): the fp32 tile of split sp of group g goes to
// C + (g*splits + sp) * gC; a second kernel adds the splits in order.
// WM x WN wavefronts tile the BM x BN block, KG k-groups share it: 64*WM*WN*KG threads.
// DB: two LDS tile buffers and one barrier per k-tile (ST = 1, KG = 1, not PERSIST): the LDS
// stores of tile i+1 and the global loads of tile i+2 are issued ahead of the MFMAs of tile i.
// bid / nblk: this workgroup's index among the nblk workgroups that share the product (the grid of a
// plain launch; a slice of it when one launch carries several products).
template <typename D, bool AK, bool BKC, int EPI, int BM, int BN, int WM, int WN, int KG, int ST, bool VEC, int KT,
          bool PERSIST, bool DB, bool SLICE>
__device__ __forceinline__ void gemm_body(const GemmArgs &a, bool vecC, int splits, int k_per_split, int tiles_x,
                                          int tiles_y, int stagger, int stagger_sleeps, int bid_, int nblk_, int xcd)
{
    // a plain launch reads its position from the hardware registers (passing them through arguments was seen to
    // cost registers: a kernel at its limit started to spill)
    const int bid = SLICE ? bid_ : (int)blockIdx.x, nblk = SLICE ? nblk_ : (int)gridDim.x;
    using M = Mma<D, KT>;
    using E = typename M::E;
    constexpr int WQ = WM * WN;
    constexpr int NT = 64 * WQ * KG;
    using TA = Tile<D, AK, BM, NT, KT>;
    using TB = Tile<D, BKC, BN, NT, KT>;
    constexpr int TM = BM / (32 * WM), TN = BN / (32 * WN);   // 32x32 MFMA tiles per wave
    constexpr int LDC = 32 * TN + 4;            // staging row pitch (floats)
    constexpr bool PIPE = DB || (D::kBytes == 2 && KG == 1 && TM * TN == 4);   // fixed MFMA / LDS-read interleave
    constexpr int TILE_BYTES = (TA::ELEMS + TB::ELEMS) * (int)sizeof(E);
    constexpr int RED_BYTES = (KG - 1) * WQ * TM * TN * 16 * 64 * 4;
    constexpr int STAGE_BYTES = WQ * 32 * LDC * 4;
    constexpr int SMEM = MaxOf<(DB ? 2 : 1) * TILE_BYTES, MaxOf<RED_BYTES, STAGE_BYTES>::v>::v;
    static_assert(M::KSTEPS % KG == 0, "k-groups must divide the MFMA k-steps of a tile");

    __shared__ __attribute__((aligned(16))) unsigned char smem[SMEM];
    E *As = reinterpret_cast<E *>(smem);
    E *Bs = As + TA::ELEMS;

    const E *Z = static_cast<const E *>(a.zeros);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int w4 = wave % WQ, kg = wave / WQ;   // position in the block tile, k-group
    const int wm = (w4 % WM) * (BM / WM), wn = (w4 / WM) * (BN / WN);
    float *fsm = reinterpret_cast<float *>(smem);

    // Block tiles are numbered n-fastest, then m, then (group, split); a workgroup takes
    // tiles t = bid, bid + nblk, ... and issues the first loads of its
    // next tile before the epilogue of the current one.
    // xcd != 0 (the launcher sets it only when 8 divides both the tile count and the grid): workgroups are handed
    // to the 8 XCDs round-robin by their index and each XCD has an L2 of its own, so the workgroups with
    // bid % 8 == x together walk one contiguous eighth of the tile list (with 8 subnets: one subnet's operands per
    // L2 instead of all of them in every L2), and within a group's tile grid the list runs down 8 rows of tiles before
    // it moves one tile to the right, so that the tiles in flight on an XCD share few operand panels.
    const int per_z = tiles_x * tiles_y;
    const int total = per_z * a.G * splits;
    int t = bid, t_step = nblk, t_end = total;
    if (xcd) {
        const int chunk = total >> 3;
        t_step = nblk >> 3;
        t = (bid & 7) * chunk + (bid >> 3);
        t_end = ((bid & 7) + 1) * chunk;
    }
    int g, gz, m0, n0, kbeg, kend;
    const E *A, *B;
    auto decode = [&](int tt) {
        gz = tt / per_z;
        const int r = tt - gz * per_z;
        g = gz / splits;
        const int sp = gz - g * splits;
        if (xcd) {
            const int band = 8 * tiles_x, bi = r / band, q = r - bi * band;
            const int rows = min(tiles_y - 8 * bi, 8);
            m0 = (8 * bi + q % rows) * BM;
            n0 = (q / rows) * BN;
        } else {
            m0 = (r / tiles_x) * BM;
            n0 = (r % tiles_x) * BN;
        }
        kbeg = sp * k_per_split;
        kend = min(a.K, kbeg + k_per_split);
        A = static_cast<const E *>(a.A) + (int64_t)g * a.gA;
        B = static_cast<const E *>(a.B) + (int64_t)g * a.gB;
    };
    decode(t);

    // One resident workgroup per CU walking many tiles: all of them would alternate between the
    // MFMA-bound main loop and the HBM-bound epilogue in lockstep, leaving each resource idle
    // half of the time.  Start them in `stagger` phase groups a fraction of a tile apart.
    if (PERSIST && DB && stagger > 1) {
        const int phase = (bid >> 3) % stagger;   // bid & 7 selects the XCD
        for (int i = 0; i < phase * stagger_sleeps; ++i) __builtin_amdgcn_s_sleep(127);
    }

    f32x16 acc[TM][TN];
    typename TA::Regs ra[ST];
    typename TB::Regs rb[ST];
    // Epilogue geometry: a lane finishes 8 consecutive columns of one row; CPR such chunks per row of the wave
    // tile, RPP rows per pass of the wave, NP passes per 32-row slice.
    constexpr int CPR = 32 * TN / 8;
    constexpr int RPP = 64 / CPR;
    constexpr int NP = 32 / RPP;
    using T = typename D::T;
    // ACCW: the update product with the old weights folded into the accumulators.  The weights of a tile are
    // requested while the previous tile's epilogue runs (into registers that the main loop needs, but no epilogue)
    // and become the accumulators' starting value -w / lr; the epilogue then has nothing to wait for:
    // w - lr dW = -lr (-w / lr + dW).  Without it every workgroup's epilogue waits for 128 KB of weights while
    // its MFMA pipe idles.  (fp32 throughout: the detour through w / lr moves a result by about 2^-22 of w,
    // against bf16's half unit in the last place of 2^-9; a weight with a zero gradient keeps its bits.)
    constexpr bool ACCW = (EPI == EPI_UPDATE_ACC);
    static_assert(!ACCW || (PERSIST && DB && KG == 1 && D::kBytes == 2), "configuration of the accumulator-resident update");
    constexpr bool PRE = (EPI == EPI_UPDATE || EPI == EPI_BWD_DATA || ACCW);
    constexpr int PD = !PRE ? 1 : (DB ? TM : ((D::kBytes == 2 && !PERSIST) ? 2 : 1));
    // Old weights (update) / activations (ReLU mask) of the chunks this lane will finish in row slice i of the
    // tile at (tg, tm0, tn0), as raw 16-byte pieces.
    auto preload = [&](int i, Pre8<T> (&dst)[NP], int tg, int tm0, int tn0) {
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int m = tm0 + wm + i * 32 + p * RPP + lane / CPR;
            const int n = tn0 + wn + 8 * (lane % CPR);
            const bool ok = vecC && kg == 0 && m < a.M && n + 8 <= a.N;
            const T *src = (EPI == EPI_UPDATE || ACCW)
                               ? static_cast<const T *>(a.C) + (int64_t)tg * a.gC + (int64_t)m * a.ldc + n
                               : static_cast<const T *>(a.mask) + (int64_t)tg * a.gMask + (int64_t)m * a.ldm + n;
            const uint4 *q = reinterpret_cast<const uint4 *>(ok ? src : reinterpret_cast<const T *>(Z));
#pragma unroll
            for (int w = 0; w < (int)(sizeof(T) / 2); ++w) dst[p].v[w] = ok ? q[w] : uint4{0, 0, 0, 0};
        }
    };
    Pre8<T> pre[PD][NP];
    auto prologue = [&]() {
#pragma unroll
        for (int s = 0; s < ST; ++s) {
            TA::template load<VEC>(ra[s], A, Z, a.sam, a.sak, m0, a.M, kbeg + s * KT, kend);
            TB::template load<VEC>(rb[s], B, Z, a.sbn, a.sbk, n0, a.N, kbeg + s * KT, kend);
        }
    };
    // The fragments of MFMA k-step q+1 are read from LDS while the MFMAs of k-step q run.
    auto compute = [&](const E *Ab, const E *Bb) {
        constexpr int QN = M::KSTEPS / KG;
        typename M::Frag fa[2][TM], fb[2][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[0][i] = TA::frag(Ab, wm + i * 32, kg, lane);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[0][j] = TB::frag(Bb, wn + j * 32, kg, lane);
#pragma unroll
        for (int q = 0; q < QN; ++q) {
            if (q + 1 < QN) {
                const int ks = (q + 1) * KG + kg;
#pragma unroll
                for (int i = 0; i < TM; ++i) fa[(q + 1) & 1][i] = TA::frag(Ab, wm + i * 32, ks, lane);
#pragma unroll
                for (int j = 0; j < TN; ++j) fb[(q + 1) & 1][j] = TB::frag(Bb, wn + j * 32, ks, lane);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j] = M::mma(fb[q & 1][j], fa[q & 1][i], acc[i][j]);
        }
        if (PIPE) {
            // instruction order for the scheduler: the first k-step's LDS reads, then every MFMA
            // followed by its share of the next k-step's reads (0x008 = MFMA, 0x100 = LDS read)
            constexpr int DS_PER = TM * (AK ? 1 : 2) + TN * (BKC ? 1 : 2);
            constexpr int DPM = (DS_PER + TM * TN - 1) / (TM * TN);
            __builtin_amdgcn_sched_group_barrier(0x100, DS_PER, 0);
#pragma unroll
            for (int q = 0; q < QN; ++q)
#pragma unroll
                for (int m = 0; m < TM * TN; ++m) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, DPM, 0);
                }
        }
    };
    // The same with the k-steps of the tile in two halves and `mid()` between them (double-buffered loop: one operand's
    // half of the next tile's LDS stores and of the requests for the tile after next goes there, the other stays in
    // front - the memory system then sees half a tile's requests every half iteration instead of a whole tile's in a
    // burst, and a half's requests are issued as soon as that half of the registers is free).
    auto compute_split = [&](const E *Ab, const E *Bb, auto &&mid) {
        constexpr int QN = M::KSTEPS / KG;
        typename M::Frag fa[2][TM], fb[2][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[0][i] = TA::frag(Ab, wm + i * 32, kg, lane);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[0][j] = TB::frag(Bb, wn + j * 32, kg, lane);
        constexpr int DS_PER = TM * (AK ? 1 : 2) + TN * (BKC ? 1 : 2);
        constexpr int DPM = (DS_PER + TM * TN - 1) / (TM * TN);
        __builtin_amdgcn_sched_group_barrier(0x100, DS_PER, 0);
#pragma unroll
        for (int q = 0; q < QN; ++q) {
            if (q + 1 < QN) {
                const int ks = (q + 1) * KG + kg;
#pragma unroll
                for (int i = 0; i < TM; ++i) fa[(q + 1) & 1][i] = TA::frag(Ab, wm + i * 32, ks, lane);
#pragma unroll
                for (int j = 0; j < TN; ++j) fb[(q + 1) & 1][j] = TB::frag(Bb, wn + j * 32, ks, lane);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j] = M::mma(fb[q & 1][j], fa[q & 1][i], acc[i][j]);
#pragma unroll
            for (int m = 0; m < TM * TN; ++m) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, DPM, 0);
            }
            if (q == (QN >= 2 ? QN / 2 - 1 : 0)) {
                __builtin_amdgcn_sched_barrier(0);
                mid();
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };
    prologue();
    if constexpr (ACCW) {
#pragma unroll
        for (int d = 0; d < TM; ++d) preload(d, pre[d], g, m0, n0);
    }

    for (;;) {
        if constexpr (ACCW) {
            // accumulators <- -w / lr.  The weights came as whole 16-byte row pieces (8 columns of a row per lane);
            // the accumulator layout wants 4 consecutive columns of row lane % 32 per register quad: through the
            // wave's own staging rows, as bf16 (row pitch 68 elements: 8-byte accesses, no two of the 32 rows
            // on the same bank pair).
            constexpr int LD16 = 32 * TN + 4;
            uint16_t *st16 = reinterpret_cast<uint16_t *>(fsm + w4 * (32 * LDC));
            const float ninv = -1.0f / a.lr;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int p = 0; p < NP; ++p) {
                    uint16_t *dst = st16 + (p * RPP + lane / CPR) * LD16 + 8 * (lane % CPR);
                    *reinterpret_cast<uint2 *>(dst) = make_uint2(pre[i][p].v[0].x, pre[i][p].v[0].y);
                    *reinterpret_cast<uint2 *>(dst + 4) = make_uint2(pre[i][p].v[0].z, pre[i][p].v[0].w);
                }
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const uint2 w = *reinterpret_cast<const uint2 *>(st16 + (lane & 31) * LD16 + 32 * j + 8 * q + 4 * (lane >> 5));
                        acc[i][j][4 * q] = ninv * __uint_as_float(w.x << 16);
                        acc[i][j][4 * q + 1] = ninv * __uint_as_float(w.x & 0xffff0000u);
                        acc[i][j][4 * q + 2] = ninv * __uint_as_float(w.y << 16);
                        acc[i][j][4 * q + 3] = ninv * __uint_as_float(w.y & 0xffff0000u);
                    }
            }
            __syncthreads();   // every wave is done with its staging rows (this and the last epilogue) before operand tiles land there
        } else {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
        }
        const int ntile = (kend - kbeg + KT - 1) / KT;

        if (DB) {
            // k-tile j waits in registers ra[j % ST] until it is stored to LDS buffer j % 2, one
            // iteration before it is used; U iterations make one period of both indices.
            constexpr int BUF = TA::ELEMS + TB::ELEMS;
            constexpr int U = (ST % 2 == 0) ? ST : 2 * ST;
            TA::store(As, ra[0]);
            TB::store(Bs, rb[0]);
            TA::template load<VEC>(ra[0], A, Z, a.sam, a.sak, m0, a.M, kbeg + ST * KT, kend);
            TB::template load<VEC>(rb[0], B, Z, a.sbn, a.sbk, n0, a.N, kbeg + ST * KT, kend);
            __syncthreads();
            auto step = [&](int it, int u) {
                E *cur = As + (u & 1) * BUF, *nxt = As + ((u & 1) ^ 1) * BUF;
                const int sg = (u + 1) % ST;
                TA::store(nxt, ra[sg]);                 // tile it+1 (zeros past the end of k)
                TB::store(nxt + TA::ELEMS, rb[sg]);
                TA::template load<VEC>(ra[sg], A, Z, a.sam, a.sak, m0, a.M, kbeg + (it + 1 + ST) * KT, kend);
                TB::template load<VEC>(rb[sg], B, Z, a.sbn, a.sbk, n0, a.N, kbeg + (it + 1 + ST) * KT, kend);
                __builtin_amdgcn_sched_barrier(0);
                compute(cur, cur + TA::ELEMS);
                __syncthreads();
            };
            if (ST == 1 && TM * TN >= 8) {   // register-bound tiles: one copy of the loop body, LDS buffer chosen at run time
                // both operands k-contiguous (the forward product): measured 414 -> 396 us per launch with the B half of
                // the stores and requests in front and the A half in the middle of the tile's MFMAs; the other
                // operand layouts do not gain (backward-data 492 -> 492 .. 506 us, update unchanged)
                if constexpr (AK && BKC && !PERSIST) {
                    for (int it = 0; it < ntile; ++it) {
                        E *cur = As + (it & 1) * BUF, *nxt = As + ((it & 1) ^ 1) * BUF;
                        TB::store(nxt + TA::ELEMS, rb[0]);     // tile it+1 (zeros past the end of k)
                        TB::template load<VEC>(rb[0], B, Z, a.sbn, a.sbk, n0, a.N, kbeg + (it + 2) * KT, kend);
                        __builtin_amdgcn_sched_barrier(0);
                        compute_split(cur, cur + TA::ELEMS, [&]() {
                            TA::store(nxt, ra[0]);
                            TA::template load<VEC>(ra[0], A, Z, a.sam, a.sak, m0, a.M, kbeg + (it + 2) * KT, kend);
                        });
                        __syncthreads();
                    }
                } else {
                    for (int it = 0; it < ntile; ++it) step(it, it & 1);
                }
            } else {
                int it0 = 0;
                for (; it0 + U <= ntile; it0 += U) {
#pragma unroll
                    for (int u = 0; u < U; ++u) step(it0 + u, u);
                }
#pragma unroll
                for (int u = 0; u < U; ++u)
                    if (it0 + u < ntile) step(it0 + u, u);
            }
        } else {
        // Main loop: whole groups of ST tiles, no branch around any load (loads past the
        // end of k are masked, not skipped), so the wait counters stay exact.
        int it0 = 0;
        for (; it0 + ST <= ntile; it0 += ST) {
#pragma unroll
            for (int s = 0; s < ST; ++s) {
                TA::store(As, ra[s]);
                TB::store(Bs, rb[s]);
                __syncthreads();
                TA::template load<VEC>(ra[s], A, Z, a.sam, a.sak, m0, a.M, kbeg + (it0 + s + ST) * KT, kend);
                TB::template load<VEC>(rb[s], B, Z, a.sbn, a.sbk, n0, a.N, kbeg + (it0 + s + ST) * KT, kend);
                __builtin_amdgcn_sched_barrier(0);   // keep the prefetch ahead of the MFMAs it overlaps with
                compute(As, Bs);
                __syncthreads();
            }
        }
        // Tail: the last ntile % ST tiles are already in registers.
        const int rem = ntile - it0;
#pragma unroll
        for (int s = 0; s < ST; ++s) {
            if (s < rem) {
                TA::store(As, ra[s]);
                TB::store(Bs, rb[s]);
                __syncthreads();
                compute(As, Bs);
                __syncthreads();
            }
        }

        }
        // ---- add the k-groups' accumulators (fixed order kg = 1, 2, ...) ----
        if (KG > 1) {
            if (kg > 0) {
                float *dst = fsm + (size_t)((kg - 1) * WQ + w4) * (TM * TN * 16 * 64);
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
#pragma unroll
                        for (int v = 0; v < 16; ++v) dst[((i * TN + j) * 16 + v) * 64 + lane] = acc[i][j][v];
            }
            __syncthreads();
            if (kg == 0) {
                for (int g2 = 1; g2 < KG; ++g2) {
                    const float *src = fsm + (size_t)((g2 - 1) * WQ + w4) * (TM * TN * 16 * 64);
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int j = 0; j < TN; ++j)
#pragma unroll
                            for (int v = 0; v < 16; ++v) acc[i][j][v] += src[((i * TN + j) * 16 + v) * 64 + lane];
                }
            }
            __syncthreads();
        }

        // ---- first loads of the next tile, so that they fly during this epilogue ----
        // (only where workgroups walk several tiles: the extra live state costs registers)
        const int cg = g, cgz = gz, cm0 = m0, cn0 = n0;
        const int tn = t + t_step;
        const bool more = PERSIST && tn < t_end;
        if (PERSIST) {
            decode(more ? tn : t);   // unconditional (a last tile re-reads its own first k-tile):
            prologue();              // a branch around loads would force the loop to drain them
        }

        if constexpr (EPI == EPI_LSE) {
            // ---- row statistics straight from the accumulators ----
            // Per 32x32 block a lane holds 16 values of ONE row (lane % 32): columns 8 (v / 4) +
            // 4 (lane / 32) + v % 4; lane ^ 32 holds the other 16.  Max and sum(exp) over the wave's
            // 32 TN columns are in-lane reductions plus one cross-lane step: no staging, no stores
            // of logits.  The bias of the block tile's columns goes through LDS as floats (the
            // operand tiles are free after the last barrier of the k-loop).
            using T = typename D::T;
            for (int c = threadIdx.x; c < BN; c += NT) {
                const int n = cn0 + c;
                fsm[c] = (a.bias && n < a.N) ? D::ld(static_cast<const T *>(a.bias) + (int64_t)cg * a.gBias + n) : 0.0f;
            }
            __syncthreads();
            const int ncol0 = cn0 + wn;   // first column of the wave tile
            if (kg == 0 && ncol0 < a.N) {
                constexpr float kLog2e = 1.4426950408889634f;
                const int half = lane >> 5, r32 = lane & 31;
                const bool full = ncol0 + 32 * TN <= a.N;
                const int blk = ncol0 / (32 * TN);
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    const int m = cm0 + wm + 32 * i + r32;
                    const int label = m < a.M ? a.y[(int64_t)cg * a.gY + m] : -1;
                    float mx = -INFINITY;
#pragma unroll
                    for (int j = 0; j < TN; ++j)
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const int c = wn + 32 * j + 8 * q + 4 * half;
                            const float4 b4 = *reinterpret_cast<const float4 *>(fsm + c);
                            const float bb[4] = {b4.x, b4.y, b4.z, b4.w};
#pragma unroll
                            for (int u = 0; u < 4; ++u) {
                                float z = fmaf(a.alpha, acc[i][j][4 * q + u], bb[u]);
                                if (!full) z = (cn0 + c + u < a.N) ? z : -INFINITY;
                                acc[i][j][4 * q + u] = z;
                                mx = fmaxf(mx, z);
                            }
                        }
                    mx = fmaxf(mx, __shfl_xor(mx, 32));
                    const float ms = mx * kLog2e;
                    float se = 0.0f;
#pragma unroll
                    for (int j = 0; j < TN; ++j)
#pragma unroll
                        for (int v = 0; v < 16; ++v) se += __builtin_amdgcn_exp2f(fmaf(acc[i][j][v], kLog2e, -ms));
                    se += __shfl_xor(se, 32);
                    if (m < a.M && half == 0 && blk < a.nb) {
                        const int64_t pi = ((int64_t)cg * a.nb + blk) * a.M + m;   // [g][block][row]: rows are the fast index
                        a.pmax[pi] = mx;
                        a.psum[pi] = se;
                    }
                    // the logit of the label: rare (one block per row), so behind a wave-uniform test
                    const int rel = label - ncol0;
                    const bool hit = rel >= 0 && rel < 32 * TN && ((rel >> 2) & 1) == half;
                    if (__builtin_amdgcn_ballot_w64(hit) != 0ull) {
                        // which of the lane's registers: block j = rel / 32, v = 4 (r / 8) + r % 4 with r = rel % 32
                        const int want = hit ? (rel >> 5) * 16 + 4 * ((rel & 31) >> 3) + (rel & 3) : -1;
                        float zl = 0.0f;
#pragma unroll
                        for (int j = 0; j < TN; ++j)
#pragma unroll
                            for (int v = 0; v < 16; ++v) zl = (16 * j + v == want) ? acc[i][j][v] : zl;
                        if (hit) a.zlabel[(int64_t)cg * a.M + m] = zl;
                    }
                }
            }
        } else {
        // ---- epilogue through LDS: each lane gets 8 consecutive columns of one row ----
        float *stage = fsm + w4 * (32 * LDC);
        // per-row inputs of the cross-entropy epilogues, fetched in one batch up front
        // the 8 columns a lane finishes are the same in every row slice: one bias fetch per tile
        float bias8[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
        if ((EPI == EPI_FWD_RELU || EPI == EPI_FWD_LOGITS) && a.bias) {
            const int n = cn0 + wn + 8 * (lane % CPR);
            const int nv = a.N - n >= 8 ? 8 : (a.N - n > 0 ? a.N - n : 0);
            if (nv > 0)
                Row8<typename D::T>::ld(static_cast<const typename D::T *>(a.bias) + (int64_t)cg * a.gBias + n,
                                        vecC && nv == 8, nv, bias8);
        }
        // EPI_DZT: per tile, the labels and log-sum-exp of the 8 samples (columns) a lane finishes, and the
        // bias of each class (row) it will meet
        int lab8[8] = {-1, -1, -1, -1, -1, -1, -1, -1};
        float ls8[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
        float brow[TM][32 / RPP];
        if (EPI == EPI_DZT) {
            const int n = cn0 + wn + 8 * (lane % CPR);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const bool ok = n + e < a.N;
                lab8[e] = ok ? a.y[(int64_t)cg * a.gY + n + e] : -1;
                ls8[e] = ok ? a.lse[(int64_t)cg * a.N + n + e] * 1.4426950408889634f : 0.0f;
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int p = 0; p < 32 / RPP; ++p) {
                    const int m = cm0 + wm + i * 32 + p * RPP + lane / CPR;
                    brow[i][p] = (a.bias && m < a.M)
                                     ? D::ld(static_cast<const typename D::T *>(a.bias) + (int64_t)cg * a.gBias + m) : 0.0f;
                }
        }
        // The old weights / activations are fetched PD row slices ahead: the loads are independent of the
        // stores of earlier chunks, which the compiler cannot know, and would otherwise each wait out a full
        // memory round trip.
        if (PRE && !ACCW) {
#pragma unroll
            for (int d = 0; d < PD; ++d)
                if (d < TM) preload(d, pre[d], cg, cm0, cn0);
        }
        // The MFMAs take the operands swapped, i.e. they produce the transposed 32x32 blocks:
        // accumulator v of block (i, j) is row 32 i + lane % 32, column 32 j + 8 (v / 4) +
        // 4 (lane / 32) + v % 4, so four consecutive registers are four consecutive columns and go
        // to the staging rows as one 16-byte LDS store.  Each wave stages through its own region:
        // the LDS executes a wave's accesses in order, no workgroup barrier is needed in here.
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            if constexpr (ACCW) {
                // The accumulators hold -w / lr + dW: the new weights w - lr dW = 0 - lr * acc (the subtraction from +0
                // keeps a zero weight with a zero gradient at +0) are final before they are staged, so
                // they go through the staging rows as bf16 (half the LDS traffic; row pitch 72 elements keeps the
                // 16-byte reads aligned) and leave as the 16-byte pieces read back.  Whole pieces only (N % 8 == 0).
                constexpr int LDH = 32 * TN + 8;
                uint16_t *st16 = reinterpret_cast<uint16_t *>(stage);
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        uint2 o;
                        o.x = f32x2_to_bf16x2(0.0f - a.lr * acc[i][j][4 * q], 0.0f - a.lr * acc[i][j][4 * q + 1]);
                        o.y = f32x2_to_bf16x2(0.0f - a.lr * acc[i][j][4 * q + 2], 0.0f - a.lr * acc[i][j][4 * q + 3]);
                        *reinterpret_cast<uint2 *>(st16 + (lane & 31) * LDH + 32 * j + 8 * q + 4 * (lane >> 5)) = o;
                    }
                // the next tile's weights, slice by slice as the accumulators of this tile's slices retire (a last
                // tile asks for its own weights again and drops them)
                preload(i, pre[i], g, m0, n0);
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int p = 0; p < 32 / RPP; ++p) {
                    const int row = p * RPP + lane / CPR, ch = lane % CPR;
                    const uint4 v = *reinterpret_cast<const uint4 *>(st16 + row * LDH + 8 * ch);
                    const int m = cm0 + wm + i * 32 + row, n = cn0 + wn + 8 * ch;
                    if (m < a.M && n < a.N)
                        *reinterpret_cast<uint4 *>(static_cast<T *>(a.C) + (int64_t)cg * a.gC + (int64_t)m * a.ldc + n) = v;
                }
                continue;
            }
            __builtin_amdgcn_wave_barrier();
            if (kg == 0) {
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        *reinterpret_cast<float4 *>(stage + (lane & 31) * LDC + 32 * j + 8 * q + 4 * (lane >> 5)) =
                            make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
            }
            __builtin_amdgcn_wave_barrier();
            if (kg == 0) {
#pragma unroll
                for (int p = 0; p < 32 / RPP; ++p) {
                    const int row = p * RPP + lane / CPR, ch = lane % CPR;
                    const float4 x = *reinterpret_cast<const float4 *>(stage + row * LDC + 8 * ch);
                    const float4 y = *reinterpret_cast<const float4 *>(stage + row * LDC + 8 * ch + 4);
                    float val[8] = {x.x, x.y, x.z, x.w, y.x, y.y, y.z, y.w};
                    if (EPI == EPI_DZT) {
                        const int m = cm0 + wm + i * 32 + row;
                        float s = epi_dzt<D>(a, cg, m, cn0 + wn + 8 * ch, val, vecC, brow[i][p], lab8, ls8);
                        if (a.pmax) {   // the CPR lanes of a row add their chunks up (all lanes of the wave are here)
                            static_assert(CPR == 4 || CPR == 8, "row groups of 4 or 8 lanes");
                            // lane ^ 1, lane ^ 2 (quad permutations), then 7 - lane within the group of 8
                            s += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, s), 0xB1, 0xF, 0xF, true));
                            s += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, s), 0x4E, 0xF, 0xF, true));
                            if (CPR == 8)
                                s += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, s), 0x141, 0xF, 0xF, true));
                            const int blk = (cn0 + wn) / (32 * TN);
                            if (ch == 0 && m < a.M && blk < a.nb) a.pmax[((int64_t)cg * a.nb + blk) * a.M + m] = s;
                        }
                    } else
                        epi8<D, EPI, PRE>(a, cg, EPI == EPI_PARTIAL ? cgz : cg, cm0 + wm + i * 32 + row, cn0 + wn + 8 * ch,
                                          val, vecC, bias8, pre[i % PD][p]);
                }
            }
            if (PRE && !ACCW && i + PD < TM) preload(i + PD, pre[i % PD], cg, cm0, cn0);
        }
        }
        if (!more) break;
        t = tn;
        if (!ACCW) __syncthreads();   // staging reads are done before the next tile's LDS stores
    }
}

// waves per SIMD the register allocator must leave room for: 2 for the 128x64 wave tile (128 accumulator
// registers), 3 for the 64x64 one (bf16 kernels)
#define IST_GEMM_BOUNDS                                                                                            \
    __launch_bounds__(64 * WM * WN * KG,                                                                           \
                      (D::kBytes != 2) ? 1 : ((BM / (32 * WM)) * (BN / (32 * WN)) >= 8) ? 2                          \
                                               : ((KG == 1 && BM >= 128) ? 3 : 1))

template <typename D, bool AK, bool BKC, int EPI, int BM, int BN, int WM, int WN, int KG, int ST, bool VEC, int KT,
          bool PERSIST = (EPI == EPI_UPDATE), bool DB = false>
__global__ IST_GEMM_BOUNDS
void k_gemm_mfma(GemmArgs a, bool vecC, int splits, int k_per_split, int tiles_x, int tiles_y, int stagger,
                 int stagger_sleeps, int xcd)
{
    gemm_body<D, AK, BKC, EPI, BM, BN, WM, WN, KG, ST, VEC, KT, PERSIST, DB, false>(
        a, vecC, splits, k_per_split, tiles_x, tiles_y, stagger, stagger_sleeps, 0, 0, xcd);
}

// Several independent products of one shape class in one launch (the weight updates of all layers of a
// small network: each alone leaves most of the chip idle while it fills and drains).  Workgroups
// first[i] .. first[i+1]-1 work on product i.
constexpr int kMaxMulti = 4;
struct GemmMulti {
    GemmArgs p[kMaxMulti];
    int first[kMaxMulti + 1];
    int tiles_x[kMaxMulti], tiles_y[kMaxMulti], vecC[kMaxMulti];
    int n;
    // optional: the bias updates of the same step (narrow layers), run by the workgroups after first[n]:
    // bias_blocks column blocks for each of the bias.G subnets (bias_blocks == 0: none)
    int bias_blocks;
    BiasArgs bias;
};

template <typename D, bool AK, bool BKC, int EPI, int BM, int BN, int WM, int WN, int KG, int ST, bool VEC, int KT,
          bool PERSIST = (EPI == EPI_UPDATE), bool DB = false>
__global__ IST_GEMM_BOUNDS
void k_gemm_mfma_multi(GemmMulti mm)
{
    if ((int)blockIdx.x >= mm.first[mm.n]) {   // whole workgroups: the barrier inside is safe
        const int e = (int)blockIdx.x - mm.first[mm.n];
        bias_update_block<D>(mm.bias, e % mm.bias_blocks, e / mm.bias_blocks);
        return;
    }
    int i = 0;
    while (i + 1 < mm.n && (int)blockIdx.x >= mm.first[i + 1]) ++i;
    const GemmArgs a = mm.p[i];
    gemm_body<D, AK, BKC, EPI, BM, BN, WM, WN, KG, ST, VEC, KT, PERSIST, DB, true>(a, mm.vecC[i] != 0, 1, a.K, mm.tiles_x[i],
                                                                                    mm.tiles_y[i], 0, 0,
                                                                                    (int)blockIdx.x - mm.first[i],
                                                                                    mm.first[i + 1] - mm.first[i], 0);
}

// out[g][m][n] = epilogue(sum_sp partial[g*splits + sp][m][n]) for split-K launches.
template <typename D, int EPI>
__global__ __launch_bounds__(256) void k_splitk_finish(GemmArgs a, const float *__restrict__ partial,
                                                       int splits, bool vecC)
{
    const int g = blockIdx.z;
    const int chunks_per_row = (a.N + 7) / 8;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (int64_t)a.M * chunks_per_row) return;
    const int m = (int)(idx / chunks_per_row), n0 = (int)(idx % chunks_per_row) * 8;
    const int nv = a.N - n0 < 8 ? a.N - n0 : 8;
    const int64_t mn = (int64_t)a.M * a.N;
    const bool pvec = (a.N % 4 == 0) && nv == 8;
    float val[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int sp = 0; sp < splits; ++sp) {
        float t[8];
        Row8<float>::ld(partial + ((int64_t)g * splits + sp) * mn + (int64_t)m * a.N + n0, pvec, nv, t);
#pragma unroll
        for (int i = 0; i < 8; ++i) val[i] += t[i];
    }
    float bias8[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
    if ((EPI == EPI_FWD_RELU || EPI == EPI_FWD_LOGITS) && a.bias)
        Row8<typename D::T>::ld(static_cast<const typename D::T *>(a.bias) + (int64_t)g * a.gBias + n0, vecC && nv == 8, nv,
                                bias8);
    epi8<D, EPI>(a, g, g, m, n0, val, vecC, bias8);
}

// 16-byte loads need an aligned base and group stride and a pitch that is a multiple
// of the chunk size.  The contiguous extent may end inside a chunk when the pitch is
// padded: along m/n the extra elements only feed output rows/columns that the epilogue
// drops, along k the padding of the library's own buffers is kept at zero.
static bool vec_ok(const void *base, int64_t gstride, int64_t pitch, int esz)
{
    const int ch = 16 / esz;
    return reinterpret_cast<uintptr_t>(base) % 16 == 0 && gstride % ch == 0 && pitch % ch == 0;
}

static bool vec_c_ok(const GemmArgs &a, int epi, int esz)
{
    const int out_esz = (epi == EPI_FWD_LOGITS || epi == EPI_PARTIAL) ? 4 : esz;
    const int ch = 16 / out_esz;
    bool ok = reinterpret_cast<uintptr_t>(a.C) % 16 == 0 && a.gC % ch == 0 && a.ldc % ch == 0;
    const int che = 16 / esz;
    if (epi == EPI_LSE) return true;   // nothing is stored, the bias is read per element
    if ((epi == EPI_FWD_RELU || epi == EPI_FWD_LOGITS) && a.bias)
        ok = ok && reinterpret_cast<uintptr_t>(a.bias) % 16 == 0 && a.gBias % che == 0;
    if (epi == EPI_BWD_DATA)
        ok = ok && reinterpret_cast<uintptr_t>(a.mask) % 16 == 0 && a.gMask % che == 0 && a.ldm % che == 0;
    return ok;
}

// Tile configuration and split-K plan as a function of the problem shape only, so that
// the workspace can be sized when the context is created.
//   tile 128: 128x128 block, 4 waves.  bf16 MFMAs are fast enough that it wins as soon as
//             it fills the chip once; f32 MFMAs are slow, there smaller blocks spread better.
//   tile 64 : 64x64 block, 4 waves x kg k-groups; kg > 1 only when there are too few blocks
//             to give every SIMD a wave.
//   tile 32 : 64x32 block (2 waves x kg), for the smallest products.
// Splitting k over workgroups costs a second kernel, so it is kept for products with a very
// long k and few tiles (the backward-data product of a very wide output layer).
SplitPlan plan_gemm(int32_t M, int32_t N, int32_t K, int32_t G, bool allow_split, int esz)
{
    constexpr int KT = 128;   // split boundaries are multiples of every k-tile size in use
    SplitPlan p{};
    p.kg = 1;
    const int64_t big_tiles = (int64_t)((M + 127) / 128) * ((N + 127) / 128) * G;
    if (big_tiles >= (esz == 2 ? 256 : 1024) && M > 64 && N > 64) {
        p.tile = 128; p.splits = 1; p.k_per_split = K; p.tiles = big_tiles;
        return p;
    }
    p.tile = 64;
    p.tiles = (int64_t)((M + 63) / 64) * ((N + 63) / 64) * G;
    int splits = 1;
    if (allow_split && esz == 2 && K >= 16384 && M > 128 && M <= 256 && N <= 128) {
        // a very long k over an output of at most one 256x128 block per group (backward-data of a wide
        // output layer): one block covers the whole output, so every operand byte is fetched once -
        // 64x64 blocks on different XCDs re-read dz twice and W four times
        p.cover = 1;
        p.tiles = G;
        const int64_t want = 1024 / p.tiles > 0 ? 1024 / p.tiles : 1;
        const int64_t most = K / (16 * KT);
        splits = (int)(want < most ? want : most);
        if (splits < 1) splits = 1;
    } else if (allow_split && p.tiles <= 256 && K >= 16384) {
        const int64_t want = 4096 / p.tiles;          // aim at ~4096 workgroups
        const int64_t most = K / (16 * KT);           // at least 16 k-tiles per split
        splits = (int)(want < most ? want : most);
        if (splits < 1) splits = 1;
    } else if (allow_split && (p.tiles <= 32 ? K >= 512 : (p.tiles <= 128 && K >= 4096))) {
        // a handful of blocks walking a long k (narrow output layer): latency-bound, spread k over the chip
        const int64_t want = 512 / p.tiles;
        const int64_t most = K / KT;
        splits = (int)(want < most ? want : most);
        if (splits < 1) splits = 1;
    }
    int kps = ((K + splits - 1) / splits + KT - 1) / KT * KT;
    if (kps < KT) kps = KT;
    splits = (K + kps - 1) / kps;
    p.splits = splits; p.k_per_split = kps;
    if (p.cover) { if (splits == 1) { p.cover = 0; p.tiles = (int64_t)((M + 63) / 64) * ((N + 63) / 64) * G; } else return p; }
    const int64_t wgs = p.tiles * splits;
    if (wgs >= 512 || K < 256) p.kg = 1;             // enough blocks (or too little k to share)
    else if (wgs <= 192 && N > 32) { p.tile = 32; p.kg = 2; }   // kg: "many", resolved per dtype
    else p.kg = 2;
    return p;
}

// Per-dtype parameters: k-tile sizes, k-groups of the small configurations and the register stages of the 64x64
// k-group kernel (measured: bf16 forward 15.1 us with 3 stages against 16.8 / 15.7 with 2 / 6; f32 45.4 us with 3
// against 44.2 with 2 and 56.4 with 6 on the 8192-wide speech model).
template <typename D> struct Cfg;
template <> struct Cfg<F32> { static constexpr int KG64 = 4, KG32 = 4, ST64 = 2, KT_SMALL = 64, KT_BIG = 32, ST_BIG = 2; };
template <> struct Cfg<BF16> { static constexpr int KG64 = 2, KG32 = 4, ST64 = 3, KT_SMALL = 64, KT_BIG = 64, ST_BIG = 1; };

// 1-D grid over block tiles.  With many more tiles than the chip holds at once the grid is
// capped and every workgroup walks several tiles (prefetching across them); otherwise one
// tile per workgroup.
static thread_local const char *s_label = "";   // product and storage type of the launch in progress
static thread_local double s_bytes = 0.0;        // its algorithmic HBM bytes

// Bytes a product has to move when every operand element is read once and every result written once
// (the update also reads the weights it rewrites; the ReLU mask of the backward-data product is read).
static double algo_bytes(const GemmArgs &a, int epi, int esz)
{
    const double G = a.G, M = a.M, N = a.N, K = a.K, e = esz;
    double b = G * (M * K + N * K) * e;
    switch (epi) {
    case EPI_FWD_RELU: b += G * M * N * e; break;
    case EPI_FWD_LOGITS: case EPI_PARTIAL: b += G * M * N * 4.0; break;
    case EPI_BWD_DATA: b += 2.0 * G * M * N * e; break;
    case EPI_UPDATE: b += 2.0 * G * M * N * e; break;
    case EPI_DZT: b += G * M * N * e; break;
    default: break;   // EPI_LSE stores only the per-block statistics
    }
    return b;
}

template <int BM, int BN, typename K>
static void launch_tiles(K kernel, int threads, const GemmArgs &a, bool vecC, int splits, int kps, hipStream_t st,
                         bool persist = false, int64_t cap = 256 * 3 * 4 /* 256 CUs x 3 resident workgroups x 4 */,
                         int stagger = 0, int stagger_sleeps = 0, bool xcd_order = false)
{
    const int tx = (a.N + BN - 1) / BN, ty = (a.M + BM - 1) / BM;
    const int64_t total = (int64_t)tx * ty * a.G * splits;
    const unsigned grid = (unsigned)(persist && total >= 4 * cap ? cap : total);
    // the per-XCD tile order needs equal shares: 8 divides the tile count and the grid (then every workgroup
    // has at least one tile of its XCD's share, since grid <= total)
    const int xcd = (xcd_order && total % 8 == 0 && grid % 8 == 0) ? 1 : 0;
    char label[64];
    snprintf(label, sizeof(label), "gemm_%s_%dx%d_t%d%s%s", s_label, BM, BN, threads, persist ? "_persistent" : "",
             splits > 1 ? "_splitk" : "");
    tag_kernel(label, 2.0 * a.M * a.N * (double)a.K * a.G, s_bytes);
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(threads), 0, st, a, vecC, splits, kps, tx, ty, stagger, stagger_sleeps, xcd);
}

template <typename D, bool AK, bool BKC, int EPI, bool VEC>
static void launch_small(const GemmArgs &a, const SplitPlan &p, bool vecC, hipStream_t st)
{
    constexpr int KTS = Cfg<D>::KT_SMALL, KG64 = Cfg<D>::KG64, KG32 = Cfg<D>::KG32;
    if (EPI == EPI_UPDATE) {
        // k = batch size is short and the block count is large: plain 64x64 blocks, 32-wide k-tiles
        launch_tiles<64, 64>(k_gemm_mfma<D, AK, BKC, EPI, 64, 64, 2, 2, 1, 3, VEC, 32>, 256, a, vecC, 1, a.K, st, true);
        return;
    }
    // (tiles ordered by XCD where 8 divides their number: a subnet's activations are then fetched by one or two L2s
    // instead of all eight; cfg3 2.013 -> 1.996 ms per round)
    if (p.tile == 32)   // double-buffered: one barrier per k-tile for the 8..16 waves of these workgroups
        launch_tiles<64, 32>(k_gemm_mfma<D, AK, BKC, EPI, 64, 32, 2, 1, KG32, 1, VEC, KTS, false, true>, 128 * KG32, a, vecC,
                             p.splits, p.k_per_split, st, false, 256 * 3 * 4, 0, 0, true);
    else if (p.kg > 1)
        launch_tiles<64, 64>(k_gemm_mfma<D, AK, BKC, EPI, 64, 64, 2, 2, KG64, Cfg<D>::ST64, VEC, KTS>, 256 * KG64, a, vecC,
                             p.splits, p.k_per_split, st, false, 256 * 3 * 4, 0, 0, true);
    else
        launch_tiles<64, 64>(k_gemm_mfma<D, AK, BKC, EPI, 64, 64, 2, 2, 1, 3, VEC, KTS>, 256, a, vecC, p.splits,
                             p.k_per_split, st, false, 256 * 3 * 4, 0, 0, true);
}

// the plan of one launch: k is split only where the epilogue allows it and the scratch buffer is large enough
static SplitPlan plan_for(const GemmArgs &a, int epi, int esz)
{
    const bool can_split = epi != EPI_UPDATE && epi != EPI_LSE && epi != EPI_DZT && a.partial != nullptr;
    SplitPlan p = plan_gemm(a.M, a.N, a.K, a.G, can_split, esz);
    if (p.splits > 1 && (size_t)a.G * p.splits * a.M * a.N * sizeof(float) > a.partial_bytes)
        p = plan_gemm(a.M, a.N, a.K, a.G, false, esz);
    return p;
}

int gemm_splits(int dtype, int epi, const GemmArgs &a)
{
    if (a.M <= 0 || a.N <= 0 || a.G <= 0) return 1;
    return plan_for(a, epi, dtype == IST_BF16 ? 2 : 4).splits;
}

template <typename D, bool AK, bool BKC, int EPI, bool VEC>
static hipError_t launch_vec(const GemmArgs &a, hipStream_t st)
{
    const int esz = D::kBytes;
    const bool vecC = vec_c_ok(a, EPI, esz);
    static const char *const kEpi[] = {"fwd_relu", "fwd_logits", "bwd_data", "update", "partial", "fwd_lse", "fwd_dzt", "update"};
    static thread_local char lab[40];
    snprintf(lab, sizeof(lab), "%s_%s%s", kEpi[EPI], esz == 2 ? "bf16" : "f32", VEC ? "" : "_novec");
    s_label = lab;
    s_bytes = algo_bytes(a, EPI, esz);
    const SplitPlan p = plan_for(a, EPI, esz);
    if (p.tile == 128) {
        constexpr int KTB = Cfg<D>::KT_BIG, STB = Cfg<D>::ST_BIG;
        // bf16 forward / backward-data: 256x128 blocks (each wave 128x64) halve the LDS traffic
        // per MFMA; the update product (both operands through transposing reads) stays 128x128
        bool done = false;
        if constexpr (D::kBytes == 2 && EPI != EPI_UPDATE) {
            // 256x256 blocks, 8 waves of 128x64, double-buffered LDS, one workgroup per CU: 128 flop per
            // byte fetched through the vector memory path, which otherwise saturates before the MFMA pipe
            if (a.K > 256 && a.M > 128 && a.N >= 256 &&
                (int64_t)((a.M + 255) / 256) * ((a.N + 255) / 256) * a.G >= 256) {
                launch_tiles<256, 256>(k_gemm_mfma<D, AK, BKC, EPI, 256, 256, 2, 4, 1, 1, VEC, 64, false, true>, 512, a, vecC,
                                       1, a.K, st, false, 256 * 3 * 4, 0, 0, true);
                done = true;
            }
        }
        if constexpr (D::kBytes == 2 && EPI == EPI_UPDATE) {
            // a wide layer with at most 128 columns per subnet (a wide output layer): 256x128 blocks, so that no
            // MFMA work is spent on columns that do not exist
            if (a.N <= 128 && a.K >= 128 && (int64_t)((a.M + 255) / 256) * a.G >= 1024) {
                launch_tiles<256, 128>(k_gemm_mfma<D, AK, BKC, EPI, 256, 128, 2, 2, 1, 1, VEC, 64, true, false>, 256, a, vecC,
                                       1, a.K, st, true, 512);
                done = true;
            }
        }
        if constexpr (D::kBytes == 2 && EPI == EPI_UPDATE) {
            // wide layers: one persistent 256x256 workgroup per CU, started in 4 phase groups
            if (!done && a.K >= 256 && (int64_t)((a.M + 255) / 256) * ((a.N + 255) / 256) * a.G >= 1024) {
                // weights in whole 16-byte pieces and a usable 1 / lr: the old weights ride in the accumulators
                bool in_acc = false;
                if constexpr (VEC) in_acc = vecC && a.N % 8 == 0 && a.lr != 0.0f && std::isfinite(1.0f / a.lr);
                if constexpr (VEC) if (in_acc)
                    launch_tiles<256, 256>(k_gemm_mfma<D, AK, BKC, EPI_UPDATE_ACC, 256, 256, 2, 4, 1, 1, VEC, 64, true, true>, 512,
                                           a, vecC, 1, a.K, st, true, 256, 4, 1);
                if (!in_acc)
                    launch_tiles<256, 256>(k_gemm_mfma<D, AK, BKC, EPI, 256, 256, 2, 4, 1, 1, VEC, 64, true, true>, 512, a, vecC,
                                           1, a.K, st, true, 256, 4, 1);
                done = true;
            }
        }
        if (done) {
        } else if (EPI != EPI_UPDATE && a.K <= 256 && p.tiles >= 4 * 3072) {
            // very short k, very many tiles (wide output layer): walk tiles persistently so that the
            // loads of the next tile overlap the (arithmetic-heavy) epilogue of the current one
            launch_tiles<128, 128>(k_gemm_mfma<D, AK, BKC, EPI, 128, 128, 2, 2, 1, STB, VEC, KTB, true>, 256, a, vecC, 1,
                                   a.K, st, true);
        } else if (D::kBytes == 2 && EPI != EPI_UPDATE && a.M > 128)
            launch_tiles<256, 128>(k_gemm_mfma<D, AK, BKC, EPI, 256, 128, 2, 2, 1, 1, VEC, 64>, 256, a, vecC, 1, a.K, st, EPI == EPI_UPDATE);
        else
            launch_tiles<128, 128>(k_gemm_mfma<D, AK, BKC, EPI, 128, 128, 2, 2, 1, STB, VEC, KTB>, 256, a, vecC, 1, a.K, st,
                                   EPI == EPI_UPDATE);
    } else if (p.splits == 1) {
        launch_small<D, AK, BKC, EPI, VEC>(a, p, vecC, st);
    } else {
        GemmArgs pa = a;
        pa.C = a.partial; pa.ldc = a.N; pa.gC = (int64_t)a.M * a.N;
        const bool vecP = vec_c_ok(pa, EPI_PARTIAL, esz);
        bool covered = false;
        if constexpr (D::kBytes == 2) {
            if (p.cover) {
                launch_tiles<256, 128>(k_gemm_mfma<D, AK, BKC, EPI_PARTIAL, 256, 128, 2, 2, 1, 1, VEC, 64>, 256, pa, vecP,
                                       p.splits, p.k_per_split, st);
                covered = true;
            }
        }
        if (!covered) launch_small<D, AK, BKC, EPI_PARTIAL, VEC>(pa, p, vecP, st);
        if (a.keep_partial) return hipGetLastError();
        const int64_t units = (int64_t)a.M * ((a.N + 7) / 8);
        dim3 g2((unsigned)((units + 255) / 256), 1, (unsigned)a.G);
        hipLaunchKernelGGL((k_splitk_finish<D, EPI>), g2, dim3(256), 0, st, a, a.partial, p.splits, vecC);
    }
    return hipGetLastError();
}

template <typename D, bool AK, bool BKC, int EPI>
static hipError_t launch_cfg(const GemmArgs &a, hipStream_t st)
{
    const int esz = D::kBytes;
    const bool vecA = vec_ok(a.A, a.gA, AK ? a.sam : a.sak, esz);
    const bool vecB = vec_ok(a.B, a.gB, BKC ? a.sbn : a.sbk, esz);
    return (vecA && vecB) ? launch_vec<D, AK, BKC, EPI, true>(a, st) : launch_vec<D, AK, BKC, EPI, false>(a, st);
}

template <typename D>
static hipError_t launch_dtype(int epi, const GemmArgs &a, hipStream_t st)
{
    // which index of an operand is contiguous follows from the product (with a 1-wide operand both
    // strides are 1 and either reading is right)
    const bool a_k = a.sak == 1, a_m = a.sam == 1, b_k = a.sbk == 1, b_n = a.sbn == 1;
    switch (epi) {
    case EPI_FWD_RELU:
        if (a_k && b_k) return launch_cfg<D, true, true, EPI_FWD_RELU>(a, st);
        break;
    case EPI_FWD_LOGITS:
        if (a_k && b_k) return launch_cfg<D, true, true, EPI_FWD_LOGITS>(a, st);
        break;
    case EPI_LSE:
        if (a_k && b_k) return launch_cfg<D, true, true, EPI_LSE>(a, st);
        break;
    case EPI_DZT:
        if (a_k && b_k) return launch_cfg<D, true, true, EPI_DZT>(a, st);
        break;
    case EPI_BWD_DATA:
        if (a_k && b_n) return launch_cfg<D, true, false, EPI_BWD_DATA>(a, st);
        if (a_m && b_n) return launch_cfg<D, false, false, EPI_BWD_DATA>(a, st);   // dz stored transposed
        break;
    case EPI_UPDATE:
        if (a_m && b_n) return launch_cfg<D, false, false, EPI_UPDATE>(a, st);
        if (a_k && b_n) return launch_cfg<D, true, false, EPI_UPDATE>(a, st);      // dz stored transposed
        break;
    default: break;
    }
    return hipErrorInvalidValue;
}

int dzt_block_width(int dtype, int32_t M, int32_t N, int32_t K, int32_t G)
{
    const SplitPlan p = plan_gemm(M, N, K, G, false, dtype == IST_BF16 ? 2 : 4);
    // 64x64 and 64x32 blocks: wave tiles 32 columns wide; 128x128, 256x128 and 256x256 blocks: 64 columns
    return p.tile == 128 ? 64 : 32;
}

int lse_block_width(int dtype, int32_t M, int32_t N, int32_t K, int32_t G)
{
    const SplitPlan p = plan_gemm(M, N, K, G, false, dtype == IST_BF16 ? 2 : 4);
    return p.tile == 128 ? 64 : 32;   // 32 * TN of the configuration launch_vec picks
}

// The update products of several layers.  Those that take the small persistent 64x64 kernel with 16-byte
// operand loads (every layer of the small f32 configurations) share one launch; any other goes out alone
// (sharing a launch among 128x128-block products was measured and gains nothing: they already fill the chip).
static bool update_shares_launch(const GemmArgs &a, int esz)
{
    if (a.M <= 0 || a.N <= 0 || a.G <= 0) return false;
    const bool layout = a.sam == 1 && a.sbn == 1 && a.sak != 1 && a.sbk != 1;
    const bool vec = vec_ok(a.A, a.gA, a.sak, esz) && vec_ok(a.B, a.gB, a.sbk, esz);
    const SplitPlan p = plan_for(a, EPI_UPDATE, esz);
    const int64_t total = (int64_t)((a.N + 63) / 64) * ((a.M + 63) / 64) * a.G;
    return layout && vec && p.tile != 128 && total <= (1 << 20);
}

bool gemm_update_shares_launch(int dtype, const GemmArgs &a)
{
    return update_shares_launch(a, dtype == IST_BF16 ? 2 : 4);
}

// bias (optional): the narrow bias updates of the step; *bias_done tells whether they rode along
template <typename D>
static hipError_t launch_updates_typed(const GemmArgs *args, int n, const BiasArgs *bias, bool *bias_done, hipStream_t st)
{
    const int esz = D::kBytes;
    GemmMulti mm{};
    double flops = 0.0, bytes = 0.0;
    for (int i = 0; i < n; ++i) {
        const GemmArgs &a = args[i];
        if (a.M <= 0 || a.N <= 0 || a.G <= 0) continue;
        const int tx = (a.N + 63) / 64, ty = (a.M + 63) / 64;
        const int64_t total = (int64_t)tx * ty * a.G;
        if (!update_shares_launch(a, esz) || mm.n == kMaxMulti) {
            hipError_t e = launch_dtype<D>(EPI_UPDATE, a, st);
            if (e != hipSuccess) return e;
            continue;
        }
        const int64_t cap = 256 * 3 * 4;
        mm.p[mm.n] = a;
        mm.tiles_x[mm.n] = tx; mm.tiles_y[mm.n] = ty;
        mm.vecC[mm.n] = vec_c_ok(a, EPI_UPDATE, esz) ? 1 : 0;
        mm.first[mm.n + 1] = mm.first[mm.n] + (int)(total >= 4 * cap ? cap : total);
        flops += 2.0 * a.M * a.N * (double)a.K * a.G;
        bytes += algo_bytes(a, EPI_UPDATE, esz);
        ++mm.n;
    }
    if (mm.n == 0) return hipGetLastError();
    const bool ride = bias && bias->njobs > 0 && bias->G > 0;
    if (mm.n == 1 && !ride) return launch_dtype<D>(EPI_UPDATE, mm.p[0], st);
    int64_t grid = mm.first[mm.n];
    if (bias && bias->njobs > 0 && bias->G > 0) {
        mm.bias = *bias;
        int blocks = 0;
        for (int j = 0; j < mm.bias.njobs; ++j) {
            mm.bias.job[j].blk0 = blocks;
            blocks += (int)((mm.bias.job[j].R + 63) / 64);
        }
        if (blocks > 0 && (int64_t)blocks * mm.bias.G < (1 << 20)) {
            mm.bias_blocks = blocks;
            grid += (int64_t)blocks * mm.bias.G;
            if (bias_done) *bias_done = true;
        }
    }
    char label[64];
    snprintf(label, sizeof(label), "gemm_update_%s_64x64_t256_persistent_x%d%s", esz == 2 ? "bf16" : "f32", mm.n,
             mm.bias_blocks ? "_bias" : "");
    tag_kernel(label, flops, bytes);
    hipLaunchKernelGGL((k_gemm_mfma_multi<D, false, false, EPI_UPDATE, 64, 64, 2, 2, 1, 3, true, 32>), dim3((unsigned)grid),
                       dim3(256), 0, st, mm);
    return hipGetLastError();
}

hipError_t launch_gemm_updates(int dtype, const GemmArgs *args, int n, const BiasArgs *bias, bool *bias_done,
                                    hipStream_t st)
{
    if (bias_done) *bias_done = false;
    for (int i = 0; i < n; ++i)
        if (args[i].zeros == nullptr) return hipErrorInvalidValue;
    return dtype == IST_BF16 ? launch_updates_typed<BF16>(args, n, bias, bias_done, st)
                             : launch_updates_typed<F32>(args, n, bias, bias_done, st);
}

// Sum of `splits` fp32 partial products laid out [g * splits + sp][M][N] followed by the backward-data epilogue
// (factor, ReLU mask, storage rounding) into a.C: the finishing pass of a product whose k was split elsewhere.
hipError_t launch_splitk_finish_bwd(int dtype, const GemmArgs &a, const float *partial, int splits, hipStream_t st)
{
    if (a.M <= 0 || a.N <= 0 || a.G <= 0) return hipSuccess;
    const int esz = dtype == IST_BF16 ? 2 : 4;
    const bool vecC = vec_c_ok(a, EPI_BWD_DATA, esz);
    const int64_t units = (int64_t)a.M * ((a.N + 7) / 8);
    dim3 grid((unsigned)((units + 255) / 256), 1, (unsigned)a.G);
    if (dtype == IST_BF16)
        hipLaunchKernelGGL((k_splitk_finish<BF16, EPI_BWD_DATA>), grid, dim3(256), 0, st, a, partial, splits, vecC);
    else
        hipLaunchKernelGGL((k_splitk_finish<F32, EPI_BWD_DATA>), grid, dim3(256), 0, st, a, partial, splits, vecC);
    return hipGetLastError();
}

hipError_t launch_gemm(int dtype, int epi, const GemmArgs &a, hipStream_t st)
{
    if (a.M <= 0 || a.N <= 0 || a.G <= 0) return hipSuccess;
    if (a.zeros == nullptr) return hipErrorInvalidValue;
    return dtype == IST_BF16 ? launch_dtype<BF16>(epi, a, st) : launch_dtype<F32>(epi, a, st);
}

}  // namespace ist
