// MFMA grouped GEMM for the subnet SGD step (gfx950).
//
//   C_g[m][n] = sum_k A_g(m,k) * B_g(n,k),   g = subnet (blockIdx.z)
//
// Each operand is either K-contiguous (rows of k values) or M-contiguous (the
// matrix is stored with k as the slow index).  The three products of a layer
// (Section 2.1 "Training Subnets": forward, back-propagation, SGD update) are
//   forward         A = h_{l-1} (K-contig)   B = W_l (K-contig)
//   backward data   A = dz_l    (K-contig)   B = W_l (M-contig: k runs over rows of W_l)
//   backward weight A = dz_l    (M-contig)   B = h_{l-1} (M-contig)
// so no operand is ever stored twice or transposed in memory.
//
// bf16: v_mfma_f32_32x32x16_bf16.  K-contiguous tiles sit in LDS as [row][k] and a
// lane's 8 consecutive k values are one 128-bit LDS read; M-contiguous tiles sit as
// [k][row] exactly as in memory and the fragment is produced by the transposing LDS
// read ds_read_b64_tr_b16 (two per fragment).
// f32: v_mfma_f32_32x32x2_f32, one value per lane and operand; both LDS layouts
// are read with plain 32-bit loads.
//
// 256 threads = 4 wavefronts in a 2x2 arrangement; macro tile BM x BN x 32.
// Global loads are 16 bytes per lane, prefetched into registers one k-tile ahead.
#include "ist_internal.h"

namespace ist {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

constexpr int KT = 32;   // k extent of one LDS tile

template <typename D> struct Mma;

template <> struct Mma<BF16> {
    using E = uint16_t;
    using Frag = bf16x8;
    static constexpr int CH = 8;          // elements per 16-byte chunk
    static constexpr int KSTEPS = KT / 16;
    static constexpr int ld_k(int) { return KT + 8; }          // [row][k] row pitch (elements)
    static constexpr int ld_m(int rows) { return rows + 16; }  // [k][row] row pitch
    __device__ static inline f32x16 mma(Frag a, Frag b, f32x16 c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
    __device__ static inline void store_k(E *lds, int row, int kc, uint4 v, int ld)
    {
        *reinterpret_cast<uint4 *>(lds + row * ld + kc * CH) = v;
    }
    __device__ static inline Frag frag_k(const E *lds, int rb, int ks, int lane, int ld)
    {
        return *reinterpret_cast<const Frag *>(lds + (rb + (lane & 31)) * ld + ks * 16 + (lane >> 5) * 8);
    }
    __device__ static inline Frag frag_m(const E *lds, int rb, int ks, int lane, int ld)
    {
        // 16-lane block: lane q supplies the address of 4 consecutive rows-elements
        // [k0 + q/4][m0 + 4*(q%4)] and receives [k0 .. k0+3][m0 + q].
        const int q = lane & 15;
        const int m0 = rb + ((lane >> 4) & 1) * 16;
        const int k0 = ks * 16 + (lane >> 5) * 8;
        const E *p0 = lds + (k0 + (q >> 2)) * ld + m0 + 4 * (q & 3);
        const E *p1 = p0 + 4 * ld;
        typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
        s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p0));
        s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p1));
        s16x8 r = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(Frag, r);
    }
};

template <> struct Mma<F32> {
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

// One operand tile: ROWS rows (m or n) by KT k values.
template <typename D, bool KCONTIG, int ROWS>
struct Tile {
    using M = Mma<D>;
    using E = typename M::E;
    static constexpr int CH = M::CH;
    static constexpr int LD = KCONTIG ? M::ld_k(ROWS) : M::ld_m(ROWS);
    static constexpr int ELEMS = KCONTIG ? ROWS * LD : KT * LD;
    static constexpr int CHUNKS = ROWS * KT / CH;
    static constexpr int PER = (CHUNKS + 255) / 256;   // chunks per thread

    struct Regs { uint4 v[PER]; };

    // chunk c -> (row, k) of its first element inside the tile
    __device__ static inline void coords(int c, int &row, int &k)
    {
        if (KCONTIG) { row = c / (KT / CH); k = (c % (KT / CH)) * CH; }
        else         { k = c / (ROWS / CH); row = (c % (ROWS / CH)) * CH; }
    }

    // s_row / s_k: element strides of the row index and of k (one of them is 1)
    __device__ static inline void load(Regs &r, const E *base, int64_t s_row, int64_t s_k, int row0,
                                       int rows_total, int k0, int K, bool vec)
    {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int c = threadIdx.x + i * 256;
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (CHUNKS % 256 == 0 || c < CHUNKS) {
                int row, k;
                coords(c, row, k);
                const int gr = row0 + row, gk = k0 + k;
                if (gr < rows_total && gk < K) {
                    const E *p = base + (int64_t)gr * s_row + (int64_t)gk * s_k;
                    if (vec) {
                        v = *reinterpret_cast<const uint4 *>(p);
                    } else {
                        E tmp[CH];
#pragma unroll
                        for (int e = 0; e < CH; ++e) {
                            const bool ok = KCONTIG ? (gk + e < K) : (gr + e < rows_total);
                            tmp[e] = ok ? p[e] : (E)0;
                        }
                        __builtin_memcpy(&v, tmp, 16);
                    }
                }
            }
            r.v[i] = v;
        }
    }

    __device__ static inline void store(E *lds, const Regs &r)
    {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int c = threadIdx.x + i * 256;
            if (CHUNKS % 256 == 0 || c < CHUNKS) {
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

template <typename D, bool AK, bool BKC, int EPI, int BM, int BN>
__global__ __launch_bounds__(256) void k_gemm_mfma(GemmArgs a, bool vecA, bool vecB)
{
    using M = Mma<D>;
    using E = typename M::E;
    using TA = Tile<D, AK, BM>;
    using TB = Tile<D, BKC, BN>;
    constexpr int TM = BM / 64, TN = BN / 64;   // 32x32 MFMA tiles per wave

    __shared__ __attribute__((aligned(16))) E As[TA::ELEMS];
    __shared__ __attribute__((aligned(16))) E Bs[TB::ELEMS];

    const int g = blockIdx.z;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const E *A = static_cast<const E *>(a.A) + (int64_t)g * a.gA;
    const E *B = static_cast<const E *>(a.B) + (int64_t)g * a.gB;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = (wave & 1) * (BM / 2), wn = (wave >> 1) * (BN / 2);

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    typename TA::Regs ra;
    typename TB::Regs rb;
    TA::load(ra, A, a.sam, a.sak, m0, a.M, 0, a.K, vecA);
    TB::load(rb, B, a.sbn, a.sbk, n0, a.N, 0, a.K, vecB);

    for (int k0 = 0; k0 < a.K; k0 += KT) {
        TA::store(As, ra);
        TB::store(Bs, rb);
        __syncthreads();
        if (k0 + KT < a.K) {
            TA::load(ra, A, a.sam, a.sak, m0, a.M, k0 + KT, a.K, vecA);
            TB::load(rb, B, a.sbn, a.sbk, n0, a.N, k0 + KT, a.K, vecB);
        }
#pragma unroll
        for (int ks = 0; ks < M::KSTEPS; ++ks) {
            typename M::Frag fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) fa[i] = TA::frag(As, wm + i * 32, ks, lane);
#pragma unroll
            for (int j = 0; j < TN; ++j) fb[j] = TB::frag(Bs, wn + j * 32, ks, lane);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j] = M::mma(fa[i], fb[j], acc[i][j]);
        }
        __syncthreads();
    }

    // ---------------- epilogue ----------------
    using T = typename D::T;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int n = n0 + wn + j * 32 + (lane & 31);
            if (n >= a.N) continue;
            float bias = 0.0f;
            if ((EPI == EPI_FWD_RELU || EPI == EPI_FWD_LOGITS) && a.bias)
                bias = D::ld(static_cast<const T *>(a.bias) + (int64_t)g * a.gBias + n);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + wm + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                if (m >= a.M) continue;
                float val = acc[i][j][v];
                const int64_t ci = (int64_t)g * a.gC + (int64_t)m * a.ldc + n;
                if (EPI == EPI_FWD_RELU) {
                    val += bias;
                    static_cast<T *>(a.C)[ci] = D::cvt(val > 0.0f ? val : 0.0f);
                } else if (EPI == EPI_FWD_LOGITS) {
                    static_cast<float *>(a.C)[ci] = val + bias;
                } else if (EPI == EPI_BWD_DATA) {
                    float h = D::ld(static_cast<const T *>(a.mask) + (int64_t)g * a.gMask + (int64_t)m * a.ldm + n);
                    static_cast<T *>(a.C)[ci] = D::cvt(h > 0.0f ? val : 0.0f);
                } else {
                    T *w = static_cast<T *>(a.C) + ci;
                    *w = D::cvt(D::up(*w) - a.lr * val);
                }
            }
        }
    }
}

// 16-byte loads need: aligned base and group stride, contiguous extent and the
// strided pitch multiples of the chunk size.
static bool vec_ok(const void *base, int64_t gstride, int64_t pitch, int64_t extent, int esz)
{
    const int ch = 16 / esz;
    return reinterpret_cast<uintptr_t>(base) % 16 == 0 && gstride % ch == 0 && pitch % ch == 0 &&
           extent % ch == 0;
}

template <typename D, bool AK, bool BKC, int EPI>
static hipError_t launch_cfg(const GemmArgs &a, hipStream_t st)
{
    const int esz = D::kBytes;
    // A: K-contig -> pitch sam, extent K; M-contig -> pitch sak, extent M
    const bool vecA = AK ? vec_ok(a.A, a.gA, a.sam, a.K, esz) : vec_ok(a.A, a.gA, a.sak, a.M, esz);
    const bool vecB = BKC ? vec_ok(a.B, a.gB, a.sbn, a.K, esz) : vec_ok(a.B, a.gB, a.sbk, a.N, esz);
    const int64_t big_tiles = (int64_t)((a.M + 127) / 128) * ((a.N + 127) / 128) * a.G;
    if (big_tiles >= 192 && a.M > 64 && a.N > 64) {
        dim3 grid((unsigned)((a.N + 127) / 128), (unsigned)((a.M + 127) / 128), (unsigned)a.G);
        hipLaunchKernelGGL((k_gemm_mfma<D, AK, BKC, EPI, 128, 128>), grid, dim3(256), 0, st, a, vecA, vecB);
    } else {
        dim3 grid((unsigned)((a.N + 63) / 64), (unsigned)((a.M + 63) / 64), (unsigned)a.G);
        hipLaunchKernelGGL((k_gemm_mfma<D, AK, BKC, EPI, 64, 64>), grid, dim3(256), 0, st, a, vecA, vecB);
    }
    return hipGetLastError();
}

template <typename D>
static hipError_t launch_dtype(int epi, const GemmArgs &a, hipStream_t st)
{
    const bool ak = a.sak == 1, bk = a.sbk == 1;
    if (!ak && a.sam != 1) return hipErrorInvalidValue;
    if (!bk && a.sbn != 1) return hipErrorInvalidValue;
    switch (epi) {
    case EPI_FWD_RELU:
        if (ak && bk) return launch_cfg<D, true, true, EPI_FWD_RELU>(a, st);
        break;
    case EPI_FWD_LOGITS:
        if (ak && bk) return launch_cfg<D, true, true, EPI_FWD_LOGITS>(a, st);
        break;
    case EPI_BWD_DATA:
        if (ak && !bk) return launch_cfg<D, true, false, EPI_BWD_DATA>(a, st);
        break;
    case EPI_UPDATE:
        if (!ak && !bk) return launch_cfg<D, false, false, EPI_UPDATE>(a, st);
        break;
    default: break;
    }
    return hipErrorInvalidValue;
}

hipError_t launch_gemm_mfma(int dtype, int epi, const GemmArgs &a, hipStream_t st)
{
    if (a.M <= 0 || a.N <= 0 || a.G <= 0) return hipSuccess;
    if ((a.M + 63) / 64 > 65535) return hipErrorInvalidValue;
    return dtype == IST_BF16 ? launch_dtype<BF16>(epi, a, st) : launch_dtype<F32>(epi, a, st);
}

}  // namespace ist
