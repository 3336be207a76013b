// Partition and merge kernels: neuron index tables, block gather/scatter.
//
// Section 2.1 "Constructing Subnets" / Appendix A of the IST paper: subnet s owns
// the block H_l^s of each hidden layer and gets W_l[H_l^s, H_{l-1}^s].  Inside a
// subnet the order of neurons does not change the function it computes, so the
// packed layout keeps each block sorted by neuron id: gathers then walk the full
// matrix in ascending address order.  ist_subnet_export undoes the sort.
#include "ist_internal.h"

namespace ist {

// 16-byte load of data that is read exactly once (a row of the full matrix on its way into the
// subnets): non-temporal, measured 6.3 .. 6.9 TB/s against 5.7 .. 6.2 TB/s for plain loads
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ inline uint4 ld_stream(const uint4 *p)
{
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
    return uint4{v.x, v.y, v.z, v.w};
}

// ----------------------------------------------------------------------------
// index tables
// ----------------------------------------------------------------------------
// The tables of up to kMaxPermJobs hidden layers are built by one launch of each of the two kernels: workgroup
// b works on the layer i with blk0[i] <= b < blk0[i + 1].
__device__ inline int perm_job_of(const int32_t *blk0, int njobs, int b)
{
    int i = 0;
    while (i + 1 < njobs && b >= blk0[i + 1]) ++i;
    return i;
}

__global__ void k_perm_invert(PermJobs jobs, int32_t *err)
{
    const int i = perm_job_of(jobs.inv_blk0, jobs.njobs, (int)blockIdx.x);
    const PermJob &j = jobs.job[i];
    int64_t p = (int64_t)((int)blockIdx.x - jobs.inv_blk0[i]) * blockDim.x + threadIdx.x;
    if (p >= j.N) return;
    int32_t c = j.perm[p];
    if (c < 0 || c >= j.N) { atomicOr(err, 1); return; }
    j.invpos[c] = (int32_t)p;
}

__global__ void k_perm_check(const int32_t *__restrict__ perm, const int32_t *__restrict__ invpos,
                             int64_t N, int32_t *err)
{
    int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= N) return;
    int32_t p = invpos[c];
    if (p < 0 || p >= N || perm[p] != (int32_t)c) atomicOr(err, 2);
}

// Ordered compaction of the neuron ids whose perm position lies in block s.  Workgroup
// (chunk j, subnet s) handles ids [1024 j, 1024 (j+1)): it first counts the members of s among
// all smaller ids (coalesced reads of the 4-byte table, no barrier inside the loop), which gives
// the packed position of its first member without any dependence on other workgroups.
constexpr int kSortThreads = 1024;
__global__ __launch_bounds__(kSortThreads) void k_perm_sort(PermJobs jobs)
{
    __shared__ int32_t wave_cnt[kSortThreads / 64];
    __shared__ int32_t wave_pre[kSortThreads / 64];
    const int ji = perm_job_of(jobs.sort_blk0, jobs.njobs, (int)blockIdx.x);
    const PermJob &job = jobs.job[ji];
    const int32_t *__restrict__ invpos = job.invpos;
    int32_t *__restrict__ sorted = job.sorted, *__restrict__ slot = job.slot, *__restrict__ p2q = job.p2q;
    uint32_t *__restrict__ mask = job.mask;
    int32_t *__restrict__ rank = job.rank;
    const int32_t S = jobs.S;
    const int64_t N = job.N, w = (N + S - 1) / S, words = (N + 31) / 32;
    const int chunk = (int)blockIdx.x - jobs.sort_blk0[ji];
    const int s = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t c0 = (int64_t)chunk * kSortThreads;
    // subnet s owns the permutation positions [p_lo, p_hi): N = q S + r, the first r blocks one wider;
    // its packed positions are s * w + 0 .. w - 1 (w = ceil(N / S)), the last one empty in a narrower block
    const int64_t qn = N / S, rn = N % S;
    const int64_t ws = qn + (s < rn ? 1 : 0);
    const int64_t p_lo = (int64_t)s * qn + (s < rn ? s : rn), p_hi = p_lo + ws;
    const int64_t pack0 = (int64_t)s * w;
    if (chunk == 0)
        for (int64_t q = ws + threadIdx.x; q < w; q += kSortThreads) sorted[pack0 + q] = -1;
    int cnt = 0;
    for (int64_t c = threadIdx.x; c < c0; c += kSortThreads) {
        const int32_t p = invpos[c];
        cnt += (p >= p_lo && p < p_hi) ? 1 : 0;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o);
    const int64_t c = c0 + threadIdx.x;
    const int32_t p = (c < N) ? invpos[c] : -1;
    const bool mine = p >= p_lo && p < p_hi;
    const unsigned long long bal = __ballot(mine);
    const int prefix = __popcll(bal & ((1ull << lane) - 1ull));
    if (lane == 0) { wave_pre[wave] = cnt; wave_cnt[wave] = __popcll(bal); }
    __syncthreads();
    int base = 0, before = 0;
    for (int i = 0; i < kSortThreads / 64; ++i) {
        base += wave_pre[i];
        before += (i < wave) ? wave_cnt[i] : 0;
    }
    if (lane == 0) {   // membership bitmask and prefix counts of these 64 neuron ids
        const int64_t w0 = (c0 + (int64_t)wave * 64) >> 5;
        const uint32_t lo = (uint32_t)bal, hi = (uint32_t)(bal >> 32);
        if (w0 < words) { mask[(int64_t)s * words + w0] = lo; rank[(int64_t)s * words + w0] = base + before; }
        if (w0 + 1 < words) {
            mask[(int64_t)s * words + w0 + 1] = hi;
            rank[(int64_t)s * words + w0 + 1] = base + before + __popc(lo);
        }
    }
    if (mine) {
        const int64_t q = (int64_t)base + before + prefix;
        if (q < ws) {   // always true for a valid permutation
            const int64_t P = pack0 + q;
            sorted[P] = (int32_t)c;
            slot[c] = (int32_t)P;
            p2q[p] = (int32_t)P;
        }
    }
}

hipError_t launch_perm_tables(PermJobs &jobs, int32_t *err, hipStream_t st)
{
    const int th = 256;
    if (jobs.njobs < 1 || jobs.njobs > kMaxPermJobs) return hipErrorInvalidValue;
    int64_t nb = 0, ns = 0;
    for (int i = 0; i < jobs.njobs; ++i) {
        jobs.inv_blk0[i] = (int32_t)nb;
        jobs.sort_blk0[i] = (int32_t)ns;
        nb += (jobs.job[i].N + th - 1) / th;
        ns += (jobs.job[i].N + kSortThreads - 1) / kSortThreads;
    }
    if (nb > 0x7fffffffLL) return hipErrorInvalidValue;
    jobs.inv_blk0[jobs.njobs] = (int32_t)nb;
    jobs.sort_blk0[jobs.njobs] = (int32_t)ns;
    hipLaunchKernelGGL(k_perm_invert, dim3((unsigned)nb), dim3(th), 0, st, jobs, err);
    hipLaunchKernelGGL(k_perm_sort, dim3((unsigned)ns, (unsigned)jobs.S), dim3(kSortThreads), 0, st, jobs);
    return hipGetLastError();
}

hipError_t launch_perm_check(const int32_t *perm, const int32_t *invpos, int64_t N, int32_t *err,
                             hipStream_t st)
{
    const int th = 256;
    hipLaunchKernelGGL(k_perm_check, dim3((unsigned)((N + th - 1) / th)), dim3(th), 0, st, perm,
                       invpos, N, err);
    return hipGetLastError();
}

// ----------------------------------------------------------------------------
// whole-row blocks (first layer: every input neuron belongs to every subnet)
// ----------------------------------------------------------------------------
// sub[P][:] <-> W[rows[P]][:], nc elements per row.  VEC: 16-byte moves.
template <typename E, bool SCATTER, bool VEC>
__global__ __launch_bounds__(256) void k_rows(E *__restrict__ W, int64_t ld, E *__restrict__ sub,
                                              const int32_t *__restrict__ rows, int64_t nrows,
                                              int64_t nc)
{
    for (int64_t P = blockIdx.x; P < nrows; P += gridDim.x) {
        const int64_t r = rows[P];
        E *pack = sub + P * nc;
        if (r < 0) {   // a packed position without a neuron (blocks of unequal width): zeros in, nothing out
            if (!SCATTER)
                for (int64_t i = threadIdx.x; i < nc; i += blockDim.x) pack[i] = E(0);
            continue;
        }
        E *full = W + r * ld;
        if (VEC) {
            constexpr int per = 16 / sizeof(E);
            const int64_t nv = nc / per;
            uint4 *f4 = reinterpret_cast<uint4 *>(full);
            uint4 *p4 = reinterpret_cast<uint4 *>(pack);
            for (int64_t i = threadIdx.x; i < nv; i += blockDim.x) {
                if (SCATTER) f4[i] = p4[i]; else p4[i] = ld_stream(f4 + i);
            }
        } else {
            for (int64_t i = threadIdx.x; i < nc; i += blockDim.x) {
                if (SCATTER) full[i] = pack[i]; else pack[i] = full[i];
            }
        }
    }
}

// Transposed first layer for sparse inputs: sub[g][c][q] <-> W[rows[g*nr+q]][c].
// 64x64 tiles staged through LDS so both sides move along their contiguous axis.
template <typename E, bool SCATTER>
__global__ __launch_bounds__(256) void k_rows_transposed(E *__restrict__ W, int64_t ld,
                                                         E *__restrict__ sub,
                                                         const int32_t *__restrict__ rows,
                                                         int64_t nr, int64_t nc)
{
    __shared__ E tile[64][65];
    const int g = blockIdx.z;
    const int64_t q0 = (int64_t)blockIdx.y * 64, c0 = (int64_t)blockIdx.x * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;   // 64 x 4
    E *pack = sub + (int64_t)g * nr * nc;                     // [nc][nr]
    if (!SCATTER) {
        for (int i = ty; i < 64; i += 4) {
            int64_t q = q0 + i, c = c0 + tx;
            if (q < nr && c < nc) {
                const int64_t r = rows[g * nr + q];   // -1: a packed position without a neuron
                tile[i][tx] = r >= 0 ? W[r * ld + c] : E(0);
            }
        }
        __syncthreads();
        for (int i = ty; i < 64; i += 4) {
            int64_t c = c0 + i, q = q0 + tx;
            if (q < nr && c < nc) pack[c * nr + q] = tile[tx][i];
        }
    } else {
        for (int i = ty; i < 64; i += 4) {
            int64_t c = c0 + i, q = q0 + tx;
            if (q < nr && c < nc) tile[tx][i] = pack[c * nr + q];
        }
        __syncthreads();
        for (int i = ty; i < 64; i += 4) {
            int64_t q = q0 + i, c = c0 + tx;
            if (q < nr && c < nc) {
                const int64_t r = rows[g * nr + q];
                if (r >= 0) W[r * ld + c] = tile[i][tx];
            }
        }
    }
}

// The same for 2-byte elements with wider accesses: a tile of 64 rows x 128 columns; the packed
// side moves 16 bytes per lane (8 consecutive q of one column), the full matrix 4 bytes per lane.
// A row of W starts at an arbitrary element (odd row lengths), so a row's aligned 4-byte words are
// staged in LDS with the row's one-element misalignment kept, and the transposing side reads
// column c of row q at position mis_q + c.  Words that straddle the tile's column range are
// written element by element on merge (their other half belongs to a neighbour).
constexpr int kTrQ = 64, kTrC = 128;
template <bool SCATTER>
__global__ __launch_bounds__(256) void k_rows_transposed16(uint16_t *__restrict__ W, int64_t ld,
                                                           uint16_t *__restrict__ sub, const int32_t *__restrict__ rows,
                                                           int64_t nr, int64_t nc, int64_t ncx, int64_t nqy, int32_t G)
{
    __shared__ uint32_t tile[kTrQ][kTrC / 2 + 2];
    __shared__ int64_t start[kTrQ];                         // element index of (row, c0) in W
    // Tiles are numbered column tile fastest, then row tile, then subnet (ncx * nqy * G of them), and the 8 XCDs
    // (workgroup index mod 8) each take one contiguous eighth of that list: a row piece of 256 bytes starts at an
    // arbitrary address, so the tiles left and right of a column boundary share a 128-byte line of every row, and as
    // neighbours on one XCD they meet it in the same L2 (the second fetch and the two partial writes of a merge stop
    // there) instead of each going to memory for it.  The grid holds 8 * ceil(tiles / 8) workgroups.
    const int64_t total = ncx * nqy * G, chunk = (total + 7) >> 3;
    const int64_t L = (int64_t)(blockIdx.x & 7) * chunk + (blockIdx.x >> 3);
    if (L >= total) return;                                 // (whole workgroups, before any barrier)
    const int64_t cx = L % ncx, rest = L / ncx;
    const int g = (int)(rest / nqy);
    const int64_t q0 = (rest % nqy) * kTrQ, c0 = cx * kTrC;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    uint16_t *pack = sub + (int64_t)g * nr * nc;            // [nc][nr]
    uint32_t *W32 = reinterpret_cast<uint32_t *>(W);
    if (threadIdx.x < kTrQ) {
        const int64_t q = q0 + threadIdx.x;
        start[threadIdx.x] = q < nr ? (int64_t)rows[g * nr + q] * ld + c0 : -1;
    }
    __syncthreads();
    const int64_t ncol = nc - c0 < kTrC ? nc - c0 : kTrC;   // valid columns of this tile
    // ---- packed side <-> LDS: thread (crow, lq) owns 8 consecutive q of one column ----
    auto packed_side = [&]() {
        const int lq = threadIdx.x & 7;
#pragma unroll
        for (int pass = 0; pass < kTrC / 32; ++pass) {
            const int crow = (threadIdx.x >> 3) + 32 * pass;
            if (crow >= ncol) continue;
            uint16_t *dst = pack + (c0 + crow) * nr + q0 + lq * 8;
            const bool full = q0 + lq * 8 + 8 <= nr;
            if (SCATTER) {
                uint16_t v[8];
                if (full) __builtin_memcpy(v, __builtin_assume_aligned(dst, 16), 16);
                else
                    for (int j = 0; j < 8; ++j) v[j] = q0 + lq * 8 + j < nr ? dst[j] : (uint16_t)0;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int qi = lq * 8 + j;
                    reinterpret_cast<uint16_t *>(tile[qi])[(start[qi] & 1) + crow] = v[j];
                }
            } else {
                uint16_t v[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int qi = lq * 8 + j;
                    v[j] = reinterpret_cast<const uint16_t *>(tile[qi])[(start[qi] & 1) + crow];
                }
                if (full) __builtin_memcpy(__builtin_assume_aligned(dst, 16), v, 16);
                else
                    for (int j = 0; j < 8; ++j)
                        if (q0 + lq * 8 + j < nr) dst[j] = v[j];
            }
        }
    };
    if (SCATTER) { packed_side(); __syncthreads(); }
    if (!SCATTER) {
        // all 16 row passes' words are requested before any is stored to LDS; a word outside the
        // tile's columns is read from word 0 of W instead (no branch around the loads)
        uint32_t v[kTrQ / 4];
#pragma unroll
        for (int pass = 0; pass < kTrQ / 4; ++pass) {
            const int64_t e0 = start[pass * 4 + ty];
            const int mis = (int)(e0 & 1);
            const int64_t lo = 2 * tx - mis;
            const int64_t e = e0 + lo;                      // first element of the word
            const bool ok = e0 >= 0 && lo < ncol;           // the row count is a multiple of 8, so W holds an
            v[pass] = W32[ok ? (e >> 1) : 0];               // even number of elements and ends on a word
        }
#pragma unroll
        for (int pass = 0; pass < kTrQ / 4; ++pass) tile[pass * 4 + ty][tx] = v[pass];
        // the 65th word of a misaligned row
        for (int i = threadIdx.x; i < kTrQ; i += 256) {
            const int64_t e0 = start[i];
            if (e0 >= 0 && (e0 & 1) && kTrC - 1 < ncol) tile[i][kTrC / 2] = W32[(e0 + kTrC - 1) >> 1];
        }
        __syncthreads();
        packed_side();
        return;
    }
    // ---- merge: LDS -> full matrix, 4 rows per pass, one aligned word per lane (+1 spill word) ----
#pragma unroll
    for (int pass = 0; pass < kTrQ / 4; ++pass) {
        const int qi = pass * 4 + ty;
        const int64_t e0 = start[qi];
        if (e0 < 0) continue;
        const int mis = (int)(e0 & 1);
        const int64_t w0 = (e0 - mis) >> 1;                 // first word of the staged range
        for (int k = tx; k < kTrC / 2 + 1; k += 64) {       // second trip: only lane 0 (word 64)
            const int64_t lo = 2 * k - mis, hi = lo + 1;    // tile columns held by word k
            if (hi < 0 || lo >= ncol) continue;
            const bool whole = lo >= 0 && hi < ncol;
            if (whole) {
                W32[w0 + k] = tile[qi][k];
            } else {
                const uint16_t *t16 = reinterpret_cast<const uint16_t *>(tile[qi]);
                if (lo >= 0 && lo < ncol) W[e0 + lo] = t16[2 * k];
                if (hi >= 0 && hi < ncol) W[e0 + hi] = t16[2 * k + 1];
            }
        }
    }
}

// ----------------------------------------------------------------------------
// column-partitioned blocks (middle and last layers)
// ----------------------------------------------------------------------------
// sub[g][i][q] <-> W[rows ? rows[g*nr+i] : i][cols[g*nc+q]].  The column lists are
// ascending, so consecutive lanes touch ascending addresses of the full row and every
// line of it is fetched once; four elements per thread are in flight.
template <typename E, bool SCATTER>
__global__ __launch_bounds__(256) void k_cols(E *__restrict__ W, int64_t ld, E *__restrict__ sub,
                                              const int32_t *__restrict__ rows,
                                              const int32_t *__restrict__ cols, int64_t nr,
                                              int64_t nc)
{
    const int g = blockIdx.z;
    const int64_t i = blockIdx.y;
    const int64_t r = rows ? (int64_t)rows[g * nr + i] : i;
    E *pack = sub + ((int64_t)g * nr + i) * nc;
    constexpr int U = 4;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    if (r < 0) {   // a packed row without a neuron (blocks of unequal width): zeros in, nothing out
        if (!SCATTER)
            for (int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; q < nc; q += stride) pack[q] = E(0);
        return;
    }
    E *full = W + r * ld;
    const int32_t *cg = cols + (int64_t)g * nc;
    for (int64_t q0 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; q0 < nc; q0 += stride * U) {
        int32_t c[U];
        E v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t q = q0 + u * stride;
            c[u] = q < nc ? cg[q] : 0;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t q = q0 + u * stride;
            if (q < nc) v[u] = SCATTER ? pack[q] : (c[u] >= 0 ? full[c[u]] : E(0));   // -1: a column without a neuron
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t q = q0 + u * stride;
            if (q < nc) { if (SCATTER) { if (c[u] >= 0) full[c[u]] = v[u]; } else pack[q] = v[u]; }
        }
    }
}

// Middle layers (rows and columns both partitioned), LDS-staged: one workgroup per packed
// row walks the source row in chunks of kMidChunk elements.  A chunk is read (and, for
// merge, written back) with 16-byte accesses along its memory order; the kept elements of
// the chunk are the contiguous range [rank(c0), rank(c0 + chunk)) of the packed row (the
// column list is ascending), so the packed side is read/written contiguously as well and
// the permutation happens in LDS.  HBM sees whole lines once in each direction.
constexpr int kMidChunk = 8192;
template <typename E, bool SCATTER>
__global__ __launch_bounds__(256) void k_mid_lds(E *__restrict__ W, int64_t ld, E *__restrict__ sub,
                                                 const int32_t *__restrict__ slotr,
                                                 const int32_t *__restrict__ cols,
                                                 const int32_t *__restrict__ rank, int64_t words, int64_t nr,
                                                 int64_t nc, int64_t N_in, int32_t G)
{
    constexpr int EPC = 16 / sizeof(E);
    constexpr int PER = kMidChunk / EPC / 256;   // 16-byte pieces per thread and chunk
    __shared__ __attribute__((aligned(16))) E buf[kMidChunk];
    // workgroups follow the rows of the full matrix, so the rows in flight are neighbours
    const int64_t P = slotr[blockIdx.x];
    if (P < 0 || P >= nr * G) return;   // only with tables built from a non-permutation
    const int g = (int)(P / nr);
    uint4 *full = reinterpret_cast<uint4 *>(W + (int64_t)blockIdx.x * ld);
    E *pack = sub + P * nc;
    const int32_t *cg = cols + (int64_t)g * nc;
    const int32_t *rg = rank + (int64_t)g * words;
    const int64_t row_pieces = N_in / EPC;
    uint4 nxt[PER];
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const int64_t c = threadIdx.x + 256 * u;
        nxt[u] = c < row_pieces ? (SCATTER ? full[c] : ld_stream(full + c)) : uint4{0, 0, 0, 0};
    }
    for (int64_t c0 = 0; c0 < N_in; c0 += kMidChunk) {
        const int64_t cend = c0 + kMidChunk < N_in ? c0 + kMidChunk : N_in;
        int64_t qlo = rg[c0 >> 5];
        int64_t qhi = cend < N_in ? rg[cend >> 5] : nc;
        qlo = qlo < 0 ? 0 : (qlo > nc ? nc : qlo);
        qhi = qhi < qlo ? qlo : (qhi > nc ? nc : qhi);
#pragma unroll
        for (int u = 0; u < PER; ++u) reinterpret_cast<uint4 *>(buf)[threadIdx.x + 256 * u] = nxt[u];
        __syncthreads();
        // the next chunk's loads fly while this one is permuted
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const int64_t c = (c0 + kMidChunk) / EPC + threadIdx.x + 256 * u;
            nxt[u] = c < row_pieces ? (SCATTER ? full[c] : ld_stream(full + c)) : uint4{0, 0, 0, 0};
        }
        for (int64_t q = qlo + threadIdx.x; q < qhi; q += 256) {
            const int64_t off = (int64_t)cg[q] - c0;
            if (off >= 0 && off < cend - c0) {   // always true for tables built from a permutation
                if (SCATTER) buf[off] = pack[q]; else pack[q] = buf[off];
            }
        }
        __syncthreads();
        if (SCATTER) {
#pragma unroll
            for (int u = 0; u < PER; ++u) {
                const int64_t c = c0 / EPC + threadIdx.x + 256 * u;
                if (c < row_pieces) full[c] = reinterpret_cast<const uint4 *>(buf)[threadIdx.x + 256 * u];
            }
            __syncthreads();
        }
    }
}

// Last layer (every row belongs to all subnets, columns partitioned): one workgroup
// per row stages the row in LDS, so that the row is read/written along its memory
// order and every packed block row is written/read as 16-byte pieces; the column
// permutation happens inside LDS.
template <typename E, bool SCATTER>
__global__ __launch_bounds__(256) void k_last_lds(E *__restrict__ W, int64_t ld, E *__restrict__ sub,
                                                  const int32_t *__restrict__ sorted, int64_t nr,
                                                  int64_t nc, int32_t G)
{
    constexpr int EPC = 16 / sizeof(E);
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    E *row = reinterpret_cast<E *>(lds_raw);
    const int64_t i = blockIdx.x;
    uint4 *full = reinterpret_cast<uint4 *>(W + i * ld);
    const int64_t nchunk = ld / EPC;
    const int64_t nunit = (int64_t)G * nc / EPC;
    if (!SCATTER) {
        for (int64_t c = threadIdx.x; c < nchunk; c += blockDim.x)
            reinterpret_cast<uint4 *>(row)[c] = ld_stream(full + c);
        __syncthreads();
        for (int64_t u = threadIdx.x; u < nunit; u += blockDim.x) {
            const int64_t P0 = u * EPC;
            const int64_t g = P0 / nc, q0 = P0 % nc;
            E e[EPC];
#pragma unroll
            for (int j = 0; j < EPC; ++j) e[j] = row[sorted[P0 + j]];
            uint4 o;
            __builtin_memcpy(&o, e, 16);
            *reinterpret_cast<uint4 *>(sub + ((int64_t)g * nr + i) * nc + q0) = o;
        }
    } else {
        for (int64_t u = threadIdx.x; u < nunit; u += blockDim.x) {
            const int64_t P0 = u * EPC;
            const int64_t g = P0 / nc, q0 = P0 % nc;
            uint4 o = *reinterpret_cast<const uint4 *>(sub + ((int64_t)g * nr + i) * nc + q0);
            E e[EPC];
            __builtin_memcpy(e, &o, 16);
#pragma unroll
            for (int j = 0; j < EPC; ++j) row[sorted[P0 + j]] = e[j];
        }
        __syncthreads();
        for (int64_t c = threadIdx.x; c < nchunk; c += blockDim.x)
            full[c] = reinterpret_cast<const uint4 *>(row)[c];
    }
}

template <typename E, bool SCATTER>
static hipError_t copy_typed(const CopyArgs &a, hipStream_t st)
{
    E *W = static_cast<E *>(a.W);
    E *sub = static_cast<E *>(a.sub);
    // bytes any kernel has to move at cache-line granularity: the rows a block touches are read
    // whole, and rewritten whole on merge when their columns are partitioned
    const double esz = sizeof(E);
    const double sub_b = (double)a.G * a.nr * a.nc * esz;
    const double rows_b = (a.rows ? (double)a.G * a.nr : (double)a.N_out) * a.N_in * esz;
    const double line_b = !a.cols ? 2.0 * sub_b
                                  : (SCATTER && a.rows ? 2.0 * rows_b + sub_b : rows_b + sub_b);
    if (a.transposed) {
        tag_kernel(SCATTER ? "k_rows_transposed<scatter>" : "k_rows_transposed<gather>", 0.0, line_b);
        if (sizeof(E) == 2 && reinterpret_cast<uintptr_t>(W) % 4 == 0 && reinterpret_cast<uintptr_t>(sub) % 16 == 0 &&
            a.nr % 8 == 0 && ((int64_t)a.nr * a.nc) % 8 == 0 && a.G * a.nr == a.N_out) {
            const int64_t ncx = (a.nc + kTrC - 1) / kTrC, nqy = (a.nr + kTrQ - 1) / kTrQ;
            const int64_t wgs = 8 * ((ncx * nqy * a.G + 7) / 8);
            if (wgs < 0x7fffffffLL) {
                hipLaunchKernelGGL((k_rows_transposed16<SCATTER>), dim3((unsigned)wgs), dim3(256), 0, st,
                                   reinterpret_cast<uint16_t *>(W), a.ld, reinterpret_cast<uint16_t *>(sub), a.rows, a.nr, a.nc,
                                   ncx, nqy, a.G);
                return hipGetLastError();
            }
        }
        dim3 grid((unsigned)((a.nc + 63) / 64), (unsigned)((a.nr + 63) / 64), (unsigned)a.G);
        hipLaunchKernelGGL((k_rows_transposed<E, SCATTER>), grid, dim3(256), 0, st, W, a.ld, sub,
                           a.rows, a.nr, a.nc);
    } else if (a.cols == nullptr) {
        const int64_t nrows = a.nr * a.G;
        const bool vec = ((a.nc * sizeof(E)) % 16 == 0) && ((a.ld * sizeof(E)) % 16 == 0) &&
                         (reinterpret_cast<uintptr_t>(W) % 16 == 0) &&
                         (reinterpret_cast<uintptr_t>(sub) % 16 == 0);
        unsigned nb = (unsigned)(nrows < 65536 ? nrows : 65536);
        tag_kernel(SCATTER ? "k_rows<scatter>" : "k_rows<gather>", 0.0, line_b);
        if (vec)
            hipLaunchKernelGGL((k_rows<E, SCATTER, true>), dim3(nb), dim3(256), 0, st, W, a.ld, sub,
                               a.rows, nrows, a.nc);
        else
            hipLaunchKernelGGL((k_rows<E, SCATTER, false>), dim3(nb), dim3(256), 0, st, W, a.ld,
                               sub, a.rows, nrows, a.nc);
    } else {
        constexpr int EPC = 16 / sizeof(E);
        const bool aligned = (reinterpret_cast<uintptr_t>(W) % 16 == 0) && (reinterpret_cast<uintptr_t>(sub) % 16 == 0) &&
                             (a.ld % EPC == 0) && (a.N_in % EPC == 0);
        const int64_t all_rows = a.nr * a.G;
        // (blocks of equal width on both sides: no packed position without a neuron)
        if (a.slotr && aligned && a.rankc && a.N_in == a.ld && a.N_in % 32 == 0 && all_rows == a.N_out &&
            a.nc * a.G == a.N_in && all_rows < 0x7fffffffLL) {
            tag_kernel(SCATTER ? "k_mid_lds<scatter>" : "k_mid_lds<gather>", 0.0, line_b);
            hipLaunchKernelGGL((k_mid_lds<E, SCATTER>), dim3((unsigned)all_rows), dim3(256), 0, st, W, a.ld, sub, a.slotr,
                               a.cols, a.rankc, a.wordsc, a.nr, a.nc, a.N_in, a.G);
            return hipGetLastError();
        }
        // the last layer's columns cover 0..N_in-1 exactly once over the G subnets
        if (!a.rows && aligned && a.nc % EPC == 0 && a.nc * a.G == a.N_in && a.N_in * sizeof(E) <= 65536 &&
            a.nr < 0x7fffffffLL) {
            int th = (int)(a.N_in / EPC);
            th = th < 64 ? 64 : (th > 256 ? 256 : (th + 63) / 64 * 64);
            tag_kernel(SCATTER ? "k_last_lds<scatter>" : "k_last_lds<gather>", 0.0, line_b);
            hipLaunchKernelGGL((k_last_lds<E, SCATTER>), dim3((unsigned)a.nr), dim3(th), (size_t)(a.N_in * sizeof(E)), st,
                               W, a.ld, sub, a.cols, a.nr, a.nc, a.G);
            return hipGetLastError();
        }
        tag_kernel(SCATTER ? "k_cols<scatter>" : "k_cols<gather>", 0.0, line_b);
        unsigned gx = (unsigned)((a.nc + 1023) / 1024);   // 4 elements per thread
        if (gx > 8) gx = 8;
        // grid.y is limited to 65535 blocks: split very tall blocks into several launches
        const int64_t max_y = 65535;
        for (int64_t i0 = 0; i0 < a.nr; i0 += max_y) {
            int64_t ny = a.nr - i0 < max_y ? a.nr - i0 : max_y;
            if (a.rows) {
                // per-group row lists are indexed by g*nr + i: this path needs nr <= max_y
                if (a.nr > max_y) return hipErrorInvalidValue;
                hipLaunchKernelGGL((k_cols<E, SCATTER>), dim3(gx, (unsigned)ny, (unsigned)a.G),
                                   dim3(256), 0, st, W, a.ld, sub, a.rows, a.cols, a.nr, a.nc);
            } else {
                for (int32_t g = 0; g < a.G; ++g)
                    hipLaunchKernelGGL((k_cols<E, SCATTER>), dim3(gx, (unsigned)ny, 1), dim3(256), 0,
                                       st, W + i0 * a.ld, a.ld,
                                       sub + ((int64_t)g * a.nr + i0) * a.nc,
                                       (const int32_t *)nullptr, a.cols + (int64_t)g * a.nc, a.nr,
                                       a.nc);
            }
        }
    }
    return hipGetLastError();
}

hipError_t launch_partition_copy(const CopyArgs &a, hipStream_t st)
{
    return a.esz == 2 ? copy_typed<uint16_t, false>(a, st) : copy_typed<uint32_t, false>(a, st);
}
hipError_t launch_merge_copy(const CopyArgs &a, hipStream_t st)
{
    return a.esz == 2 ? copy_typed<uint16_t, true>(a, st) : copy_typed<uint32_t, true>(a, st);
}

// ----------------------------------------------------------------------------
// re-sampling between rounds: merge of the old partition and partition by the new permutation in
// one pass over the full matrix (the row that merge writes is the row partition would read back)
// ----------------------------------------------------------------------------
// first layer: W[r][:] = old[slot_old[r]][:], new[slot_new[r]][:] = the same row
template <typename E>
__global__ __launch_bounds__(256) void k_resample_rows(E *__restrict__ W, int64_t ld, const E *__restrict__ sub_old,
                                                       E *__restrict__ sub_new, const int32_t *__restrict__ slot_old,
                                                       const int32_t *__restrict__ slot_new, int64_t nrows, int64_t nc)
{
    for (int64_t r = blockIdx.x; r < nrows; r += gridDim.x) {
        const int64_t Po = slot_old[r], Pn = slot_new[r];
        if (Po < 0 || Po >= nrows || Pn < 0 || Pn >= nrows) continue;   // only with non-permutation tables
        const uint4 *src = reinterpret_cast<const uint4 *>(sub_old + Po * nc);
        uint4 *full = reinterpret_cast<uint4 *>(W + r * ld);
        uint4 *dst = reinterpret_cast<uint4 *>(sub_new + Pn * nc);
        const int64_t n16 = nc * (int64_t)sizeof(E) / 16;
        for (int64_t c = threadIdx.x; c < n16; c += 256) {
            const uint4 v = src[c];
            full[c] = v;
            dst[c] = v;
        }
    }
}

// middle layers: k_mid_lds with both directions on the staged chunk
template <typename E>
__global__ __launch_bounds__(256) void k_resample_mid(E *__restrict__ W, int64_t ld, const E *__restrict__ sub_old,
                                                      E *__restrict__ sub_new, const int32_t *__restrict__ slotr_old,
                                                      const int32_t *__restrict__ slotr_new,
                                                      const int32_t *__restrict__ cols_old,
                                                      const int32_t *__restrict__ cols_new,
                                                      const int32_t *__restrict__ rank_old,
                                                      const int32_t *__restrict__ rank_new, int64_t words, int64_t nr,
                                                      int64_t nc, int64_t N_in, int32_t G)
{
    constexpr int EPC = 16 / sizeof(E);
    constexpr int PER = kMidChunk / EPC / 256;
    __shared__ __attribute__((aligned(16))) E buf[kMidChunk];
    const int64_t Po = slotr_old[blockIdx.x], Pn = slotr_new[blockIdx.x];
    if (Po < 0 || Po >= nr * G || Pn < 0 || Pn >= nr * G) return;
    const int go = (int)(Po / nr), gn = (int)(Pn / nr);
    uint4 *full = reinterpret_cast<uint4 *>(W + (int64_t)blockIdx.x * ld);
    const E *pack_old = sub_old + Po * nc;
    E *pack_new = sub_new + Pn * nc;
    const int32_t *co = cols_old + (int64_t)go * nc, *cn = cols_new + (int64_t)gn * nc;
    const int32_t *ro = rank_old + (int64_t)go * words, *rn = rank_new + (int64_t)gn * words;
    const int64_t row_pieces = N_in / EPC;
    auto clampq = [&](int64_t q) { return q < 0 ? (int64_t)0 : (q > nc ? nc : q); };
    uint4 nxt[PER];
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const int64_t c = threadIdx.x + 256 * u;
        nxt[u] = c < row_pieces ? full[c] : uint4{0, 0, 0, 0};
    }
    for (int64_t c0 = 0; c0 < N_in; c0 += kMidChunk) {
        const int64_t cend = c0 + kMidChunk < N_in ? c0 + kMidChunk : N_in;
        const int64_t qlo_o = clampq(ro[c0 >> 5]), qhi_o = cend < N_in ? clampq(ro[cend >> 5]) : nc;
        const int64_t qlo_n = clampq(rn[c0 >> 5]), qhi_n = cend < N_in ? clampq(rn[cend >> 5]) : nc;
#pragma unroll
        for (int u = 0; u < PER; ++u) reinterpret_cast<uint4 *>(buf)[threadIdx.x + 256 * u] = nxt[u];
        __syncthreads();
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const int64_t c = (c0 + kMidChunk) / EPC + threadIdx.x + 256 * u;
            nxt[u] = c < row_pieces ? full[c] : uint4{0, 0, 0, 0};
        }
        for (int64_t q = qlo_o + threadIdx.x; q < qhi_o; q += 256) {
            const int64_t off = (int64_t)co[q] - c0;
            if (off >= 0 && off < cend - c0) buf[off] = pack_old[q];
        }
        __syncthreads();
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const int64_t c = c0 / EPC + threadIdx.x + 256 * u;
            if (c < row_pieces) full[c] = reinterpret_cast<const uint4 *>(buf)[threadIdx.x + 256 * u];
        }
        for (int64_t q = qlo_n + threadIdx.x; q < qhi_n; q += 256) {
            const int64_t off = (int64_t)cn[q] - c0;
            if (off >= 0 && off < cend - c0) pack_new[q] = buf[off];
        }
        __syncthreads();
    }
}

template <typename E>
static bool resample_typed(const CopyArgs &o, const CopyArgs &n, hipStream_t st)
{
    constexpr int EPC = 16 / sizeof(E);
    E *W = static_cast<E *>(o.W);
    const E *so = static_cast<const E *>(o.sub);
    E *sn = static_cast<E *>(n.sub);
    const bool aligned = reinterpret_cast<uintptr_t>(W) % 16 == 0 && reinterpret_cast<uintptr_t>(so) % 16 == 0 &&
                         reinterpret_cast<uintptr_t>(sn) % 16 == 0 && o.ld % EPC == 0 && o.N_in % EPC == 0;
    if (o.transposed || !aligned) return false;
    const double esz = sizeof(E);
    const double sub_b = (double)o.G * o.nr * o.nc * esz, full_b = (double)o.N_out * o.N_in * esz;
    if (!o.cols) {   // first layer
        if (!o.slotr || !n.slotr || o.nc % EPC || o.nr * o.G != o.N_out) return false;
        tag_kernel("k_resample_rows", 0.0, 3.0 * sub_b);
        const int64_t nrows = o.N_out;
        hipLaunchKernelGGL((k_resample_rows<E>), dim3((unsigned)(nrows < 65536 ? nrows : 65536)), dim3(256), 0, st, W, o.ld,
                           so, sn, o.slotr, n.slotr, nrows, o.nc);
        return true;
    }
    const int64_t all_rows = o.nr * o.G;
    if (o.rows) {    // middle layer
        if (!(o.slotr && n.slotr && o.rankc && n.rankc && o.N_in == o.ld && o.N_in % 32 == 0 && all_rows == o.N_out &&
              o.nc * o.G == o.N_in && all_rows < 0x7fffffffLL))
            return false;
        tag_kernel("k_resample_mid", 0.0, 2.0 * full_b + 2.0 * sub_b);
        hipLaunchKernelGGL((k_resample_mid<E>), dim3((unsigned)all_rows), dim3(256), 0, st, W, o.ld, so, sn, o.slotr, n.slotr,
                           o.cols, n.cols, o.rankc, n.rankc, o.wordsc, o.nr, o.nc, o.N_in, o.G);
        return true;
    }
    // last layer: every line of W is owned, merge and partition each move it once already, and one
    // workgroup touching the blocks of both buffers in all S subnets measured slower than the two passes
    return false;
}

// Fused merge(old) + partition(new) of one layer; *fused = false when the shape is not covered and
// the caller has to run the two copies one after the other.
hipError_t launch_resample_copy(const CopyArgs &o, const CopyArgs &n, bool *fused, hipStream_t st)
{
    *fused = o.esz == 2 ? resample_typed<uint16_t>(o, n, st) : resample_typed<uint32_t>(o, n, st);
    return hipGetLastError();
}

// ----------------------------------------------------------------------------
// output bias: replicate on partition, mean on merge
// ----------------------------------------------------------------------------
template <typename E>
__global__ void k_bias_replicate(const E *__restrict__ b, E *__restrict__ sub, int64_t n, int32_t G)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    E v = b[i];
    for (int g = 0; g < G; ++g) sub[(int64_t)g * n + i] = v;
}

// Sum of up to 64 values as a balanced pairwise tree over the index (neighbours first, then pairs
// of pairs, ...); missing leaves are +0, which leaves every partial sum unchanged.
template <typename F>
__device__ inline float tree_sum64(int count, F value)
{
    float v[64];
#pragma unroll
    for (int s = 0; s < 64; ++s) v[s] = s < count ? value(s) : 0.0f;
#pragma unroll
    for (int d = 1; d < 64; d *= 2)
#pragma unroll
        for (int s = 0; s + d < 64; s += 2 * d) v[s] = v[s] + v[s + d];
    return v[0];
}

// b[i] = (pairwise-tree sum over the G subnet copies) * (1/G).  With G a power of two and
// identical copies every step is exact: merging an untrained partition returns the bias bit for
// bit.  Two tree levels of 64 cover G <= 4096.
template <typename D>
__global__ void k_bias_mean(typename D::T *__restrict__ b, const typename D::T *__restrict__ sub,
                            int64_t n, int32_t G)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    float acc;
    if (G <= 64) {
        acc = tree_sum64(G, [&](int s) { return D::ld(sub + (int64_t)s * n + i); });
    } else {
        const int chunks = (G + 63) / 64;
        acc = tree_sum64(chunks, [&](int c) {
            const int left = G - 64 * c;
            return tree_sum64(left < 64 ? left : 64, [&](int s) { return D::ld(sub + (int64_t)(64 * c + s) * n + i); });
        });
    }
    b[i] = D::cvt(acc * (1.0f / (float)G));
}

// hidden biases travel with their neuron: sub[P] <-> b[rows[P]]
template <typename E, bool SCATTER>
__global__ void k_bias_rows(E *__restrict__ b, E *__restrict__ sub, const int32_t *__restrict__ rows, int64_t n)
{
    const int64_t P = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (P >= n) return;
    const int32_t r = rows[P];   // -1: a packed position without a neuron
    if (SCATTER) { if (r >= 0) b[r] = sub[P]; } else sub[P] = r >= 0 ? b[r] : E(0);
}

hipError_t launch_bias_rows(void *b, void *sub, const int32_t *rows, int64_t n, int esz, bool scatter, hipStream_t st)
{
    const dim3 grid((unsigned)((n + 255) / 256));
    if (esz == 2) {
        if (scatter) hipLaunchKernelGGL((k_bias_rows<uint16_t, true>), grid, dim3(256), 0, st, (uint16_t *)b, (uint16_t *)sub, rows, n);
        else hipLaunchKernelGGL((k_bias_rows<uint16_t, false>), grid, dim3(256), 0, st, (uint16_t *)b, (uint16_t *)sub, rows, n);
    } else {
        if (scatter) hipLaunchKernelGGL((k_bias_rows<uint32_t, true>), grid, dim3(256), 0, st, (uint32_t *)b, (uint32_t *)sub, rows, n);
        else hipLaunchKernelGGL((k_bias_rows<uint32_t, false>), grid, dim3(256), 0, st, (uint32_t *)b, (uint32_t *)sub, rows, n);
    }
    return hipGetLastError();
}

hipError_t launch_bias_replicate(const void *b, void *sub, int64_t n, int32_t G, int esz,
                                 hipStream_t st)
{
    dim3 grid((unsigned)((n + 255) / 256));
    if (esz == 2)
        hipLaunchKernelGGL(k_bias_replicate<uint16_t>, grid, dim3(256), 0, st, (const uint16_t *)b,
                           (uint16_t *)sub, n, G);
    else
        hipLaunchKernelGGL(k_bias_replicate<uint32_t>, grid, dim3(256), 0, st, (const uint32_t *)b,
                           (uint32_t *)sub, n, G);
    return hipGetLastError();
}

// The bias copies of all layers of one phase in one launch: per job either sub[P] <-> b[rows[P]] (hidden
// layers, n = S * w values) or the replication of the n output biases to the G subnets (rows == null).
template <typename E, bool SCATTER>
__global__ __launch_bounds__(256) void k_bias_jobs(BiasCopyJobs a)
{
    int j = 0;
    while (j + 1 < a.njobs && (int)blockIdx.x >= a.job[j + 1].blk0) ++j;
    const BiasCopyJob jb = a.job[j];
    const int64_t i = (int64_t)(blockIdx.x - jb.blk0) * 256 + threadIdx.x;
    if (i >= jb.n) return;
    E *b = static_cast<E *>(jb.b), *sub = static_cast<E *>(jb.sub);
    if (jb.rows) {
        const int32_t r = jb.rows[i];   // -1: a packed position without a neuron
        if (SCATTER) { if (r >= 0) b[r] = sub[i]; } else sub[i] = r >= 0 ? b[r] : E(0);
    } else if (!SCATTER) {
        const E v = b[i];
        for (int g = 0; g < jb.G; ++g) sub[(int64_t)g * jb.n + i] = v;
    }
}

hipError_t launch_bias_jobs(BiasCopyJobs &a, int esz, bool scatter, hipStream_t st)
{
    int blocks = 0;
    for (int j = 0; j < a.njobs; ++j) {
        a.job[j].blk0 = blocks;
        blocks += (int)((a.job[j].n + 255) / 256);
    }
    if (blocks == 0) return hipSuccess;
    const dim3 grid((unsigned)blocks);
    if (esz == 2) {
        if (scatter) hipLaunchKernelGGL((k_bias_jobs<uint16_t, true>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((k_bias_jobs<uint16_t, false>), grid, dim3(256), 0, st, a);
    } else {
        if (scatter) hipLaunchKernelGGL((k_bias_jobs<uint32_t, true>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((k_bias_jobs<uint32_t, false>), grid, dim3(256), 0, st, a);
    }
    return hipGetLastError();
}

hipError_t launch_bias_mean(void *b, const void *sub, int64_t n, int32_t G, int dtype,
                            hipStream_t st)
{
    dim3 grid((unsigned)((n + 255) / 256));
    if (dtype == IST_BF16)
        hipLaunchKernelGGL(k_bias_mean<BF16>, grid, dim3(256), 0, st, (uint16_t *)b,
                           (const uint16_t *)sub, n, G);
    else
        hipLaunchKernelGGL(k_bias_mean<F32>, grid, dim3(256), 0, st, (float *)b, (const float *)sub,
                           n, G);
    return hipGetLastError();
}

// ----------------------------------------------------------------------------
// export one subnet block in permutation order
// ----------------------------------------------------------------------------
template <typename E>
__global__ void k_export(const E *__restrict__ sub, E *__restrict__ dst, int64_t nr, int64_t nc, int64_t pr, int64_t pc,
                         const int32_t *__restrict__ p2q_r, int64_t perm_r, int64_t pack_r,
                         const int32_t *__restrict__ p2q_c, int64_t perm_c, int64_t pack_c, bool transposed)
{
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= nr * nc) return;
    int64_t i = idx / nc, j = idx % nc;
    int64_t qi = p2q_r ? (int64_t)p2q_r[perm_r + i] - pack_r : i;
    int64_t qj = p2q_c ? (int64_t)p2q_c[perm_c + j] - pack_c : j;
    if (qi < 0 || qi >= pr || qj < 0 || qj >= pc) return;
    dst[idx] = transposed ? sub[qj * pr + qi] : sub[qi * pc + qj];
}

hipError_t launch_export(const void *sub, void *dst, int64_t nr, int64_t nc, int64_t pr, int64_t pc,
                         const int32_t *p2q_r, int64_t perm_r, int64_t pack_r, const int32_t *p2q_c,
                         int64_t perm_c, int64_t pack_c, bool transposed, int esz, hipStream_t st)
{
    int64_t n = nr * nc;
    if (n == 0) return hipSuccess;
    dim3 grid((unsigned)((n + 255) / 256));
    if (esz == 2)
        hipLaunchKernelGGL(k_export<uint16_t>, grid, dim3(256), 0, st, (const uint16_t *)sub, (uint16_t *)dst, nr, nc, pr,
                           pc, p2q_r, perm_r, pack_r, p2q_c, perm_c, pack_c, transposed);
    else
        hipLaunchKernelGGL(k_export<uint32_t>, grid, dim3(256), 0, st, (const uint32_t *)sub, (uint32_t *)dst, nr, nc, pr,
                           pc, p2q_r, perm_r, pack_r, p2q_c, perm_c, pack_c, transposed);
    return hipGetLastError();
}

}  // namespace ist
