// Internal declarations of the IST library (host plan + kernel launchers).
// gfx950 only.  Nothing here is shared with the CPU oracle.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "ist.h"

namespace ist {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// ----------------------------------------------------------------- storage types
struct F32 {
    using T = float;
    static constexpr int kBytes = 4;
    __device__ static inline float ld(const T *p) { return *p; }
    __device__ static inline T cvt(float v) { return v; }
    __device__ static inline float up(T v) { return v; }
};

__device__ inline float bf16_to_f32(uint16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
__device__ inline uint16_t f32_to_bf16(float f) {  // round to nearest even (v_cvt_pk_bf16_f32)
    return __builtin_bit_cast(uint16_t, (__bf16)f);
}
typedef __bf16 ist_bf16x2 __attribute__((ext_vector_type(2)));
typedef float ist_f32x2 __attribute__((ext_vector_type(2)));
__device__ inline uint32_t f32x2_to_bf16x2(float lo, float hi) {  // lo in bits 0..15
    ist_f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, ist_bf16x2));
}

struct BF16 {
    using T = uint16_t;
    static constexpr int kBytes = 2;
    __device__ static inline float ld(const T *p) { return bf16_to_f32(*p); }
    __device__ static inline T cvt(float v) { return f32_to_bf16(v); }
    __device__ static inline float up(T v) { return bf16_to_f32(v); }
};

// ----------------------------------------------------------------- host plan
struct LayerPlan {           // weight matrix l = 1..t
    int64_t N_out = 0, N_in = 0;   // full sizes N_l, N_{l-1}
    int64_t R = 0, C = 0;          // rows/cols held by one subnet
    int64_t ldr = 0;               // row pitch of the [B][R] activation / gradient buffers (R rounded up to 8)
    bool row_part = false;         // rows follow the blocks of hidden layer l
    bool col_part = false;         // cols follow the blocks of hidden layer l-1
    bool transposed = false;       // stored [S][C][R] (sparse-input first layer)
    size_t off_W = 0, off_b = 0;   // byte offsets into the subnet buffer
    size_t off_act = 0;            // workspace: h_l [S][maxB][R] dtype (l < t), logits fp32 (l == t)
    size_t off_dz = 0;             // workspace: dz_l [S][maxB][R] dtype
    // with per-neuron standardisation (hidden layers only):
    size_t off_z = 0;              // workspace: z_l  [S][maxB][ldr] fp32, input of the standardisation
    size_t off_zh = 0;             // workspace: zh_l [S][maxB][ldr] dtype, standardised value before the ReLU
    size_t off_isg = 0;            // workspace: 1/sigma [S][ldr] fp32
};

struct HiddenPlan {          // hidden layer l = 1..t-1
    // N = q S + r neurons: the first r subnets own q + 1, the others q.  Every subnet's block is kept in
    // w = ceil(N / S) packed positions; a position beyond the subnet's own width holds no neuron (its
    // entry in `sorted` is -1, its weights and bias are zeros, which makes it inert in the local steps).
    int64_t N = 0, w = 0;
    int64_t width(int s, int S) const { return N / S + (s < N % S ? 1 : 0); }
    int64_t perm_start(int s, int S) const { return (int64_t)s * (N / S) + (s < N % S ? s : N % S); }
    size_t off_sorted = 0;   // subnet buffer: int32 [S * w]  neuron id at sorted position P = s * w + q, or -1
    size_t off_slot = 0;     // subnet buffer: int32 [N]  sorted position of neuron id
    size_t off_p2q = 0;      // subnet buffer: int32 [N]  sorted position of perm position p
    size_t off_mask = 0;     // subnet buffer: uint32 [S][words] bit c%32 of word c/32: neuron c is in subnet s
    size_t off_rank = 0;     // subnet buffer: int32 [S][words]  neurons of subnet s below 32*word
    int64_t words = 0;       // ceil(N / 32)
    size_t off_invpos = 0;   // workspace:     int32 [N]  perm position of neuron id
};

}  // namespace ist

struct ist_ctx {
    int32_t t = 0, S = 0, dtype = 0, input = 0, has_bias = 0, max_B = 0, normalize = 0;
    float norm_eps = 1e-5f;
    std::vector<int64_t> dims;
    std::vector<float> scale;             // index l-1: factor of the product of layer l (1 without layer_scale)
    std::vector<ist::LayerPlan> layer;    // index l-1
    std::vector<ist::HiddenPlan> hidden;  // index l-1, l = 1..t-1
    size_t subnets_bytes = 0, workspace_bytes = 0;
    size_t off_rowloss = 0, off_bitmap = 0, off_err = 0;  // workspace
    size_t off_partial = 0, partial_bytes = 0, off_zeros = 0;
    bool fused_out = false;   // wide output layer: logits are never stored
    bool wide_out = false;    // ... and its part of a step runs in the two persistent launches of ist_wideout.hip
    int32_t wide_nb = 0;      // workgroups per subnet there
    size_t off_pmax = 0, off_psum = 0, off_qmax = 0, off_qsum = 0, off_zlabel = 0, off_lse = 0, off_rsum = 0; int32_t nb_max = 0;
    char *subnets = nullptr;
    char *spare = nullptr;      // second subnet buffer: target of ist_resample, then swapped in
    char *workspace = nullptr;
    bool bound = false, partitioned = false;
    int32_t checked = 0;
    std::string err;

    // optional per-launch timing (HIP events around every launch)
    struct ProfRec { int cls; hipEvent_t start, stop; char kernel[64]; double flops, bytes; };
    bool prof_on = false;
    std::vector<ProfRec> prof_recs;
    std::vector<hipEvent_t> prof_free;

    int esz() const { return dtype == IST_BF16 ? 2 : 4; }
    int32_t *errflag() const { return reinterpret_cast<int32_t *>(workspace + off_err); }
};

namespace ist {

enum KernelClass {
    KC_PERM_TABLES = 0, KC_PARTITION_COPY, KC_MERGE_COPY, KC_BIAS_COPY, KC_GEMM_FWD, KC_GEMM_BWD_DATA,
    KC_GEMM_UPDATE, KC_SOFTMAX_XENT, KC_LOSS_REDUCE, KC_BIAS_UPDATE, KC_CSR_FORWARD, KC_CSR_UPDATE,
    KC_NORM, KC_RESAMPLE, KC_COUNT
};

// What the last launcher call ran: kernel label (launch configuration), algorithmic flops and
// bytes of that launch.  Written by the launchers, read by the profiling hooks of the API.
struct KernelTag { char kernel[64]; double flops, bytes; };
extern thread_local KernelTag g_tag;
void tag_kernel(const char *label, double flops, double bytes);

// ----------------------------------------------------------------- partition / merge
// Block tables of several hidden layers (N neurons each, S blocks) from their permutations, two launches for
// all of them: invpos = inverse permutation (scratch), then per block the neuron ids sorted ascending (sorted),
// each neuron's packed position (slot), packed position by permutation position (p2q), membership bitmask per
// block (mask) and the count of members before each 32-neuron word (rank).  Fills in the blk0 fields itself.
constexpr int kMaxPermJobs = 8;
struct PermJob {
    const int32_t *perm; int32_t *invpos, *sorted, *slot, *p2q; uint32_t *mask; int32_t *rank; int64_t N;
};
struct PermJobs { PermJob job[kMaxPermJobs]; int32_t inv_blk0[kMaxPermJobs + 1], sort_blk0[kMaxPermJobs + 1]; int32_t njobs, S; };
hipError_t launch_perm_tables(PermJobs &jobs, int32_t *err, hipStream_t st);

// out[g][i][j] = W[rows ? rows[g*nr+i] : i][cols ? cols[g*nc+j] : j]  (or the
// reverse copy when scatter is set); transposed: the subnet block is [nc][nr].
struct CopyArgs {
    void *W;                 // full matrix, row-major, ld = N_in
    int64_t ld;
    void *sub;               // packed blocks [G][nr][nc] (or [G][nc][nr])
    const int32_t *rows;     // sorted neuron ids of the row layer, or null
    const int32_t *cols;     // sorted neuron ids of the col layer, or null
    const int32_t *slotr;    // sorted position of each row-layer neuron, or null
    const int32_t *slotc;    // sorted position of each col-layer neuron, or null
    const uint32_t *maskc;   // per-subnet membership bitmask of the col layer, or null
    const int32_t *rankc;    // per-subnet prefix counts matching maskc
    int64_t wordsc;          // words per subnet in maskc / rankc
    int64_t nr, nc;          // rows/cols per subnet block
    int64_t N_out, N_in;     // full sizes
    int32_t G;
    int esz;
    bool transposed;
};
hipError_t launch_partition_copy(const CopyArgs &a, hipStream_t st);
hipError_t launch_merge_copy(const CopyArgs &a, hipStream_t st);
hipError_t launch_resample_copy(const CopyArgs &old_part, const CopyArgs &new_part, bool *fused, hipStream_t st);
// bias copies of several layers in one launch (partition: gather / replicate; merge: scatter of the hidden layers)
struct BiasCopyJob { void *b; void *sub; const int32_t *rows; int64_t n; int32_t G; int32_t blk0; };
struct BiasCopyJobs { BiasCopyJob job[16]; int32_t njobs; };
hipError_t launch_bias_jobs(BiasCopyJobs &a, int esz, bool scatter, hipStream_t st);
hipError_t launch_bias_rows(void *b, void *sub, const int32_t *rows, int64_t n, int esz, bool scatter,
                            hipStream_t st);
hipError_t launch_bias_replicate(const void *b, void *sub, int64_t n, int32_t G, int esz,
                                 hipStream_t st);
hipError_t launch_bias_mean(void *b, const void *sub, int64_t n, int32_t G, int dtype,
                            hipStream_t st);
// dst[i][j], i < nr, j < nc (the subnet's own widths, permutation order) from the packed block whose
// rows / columns have pitch pr / pc positions; perm_r / pack_r: first permutation position and first
// packed position of the subnet's row block (likewise for columns); null table = identity
hipError_t launch_export(const void *sub, void *dst, int64_t nr, int64_t nc, int64_t pr, int64_t pc,
                         const int32_t *p2q_r, int64_t perm_r, int64_t pack_r, const int32_t *p2q_c,
                         int64_t perm_c, int64_t pack_c, bool transposed, int esz, hipStream_t st);

// ----------------------------------------------------------------- training
enum Epilogue {
    EPI_FWD_RELU = 0, EPI_FWD_LOGITS = 1, EPI_BWD_DATA = 2, EPI_UPDATE = 3, EPI_PARTIAL = 4,
    EPI_LSE = 5,   // logits are not stored: per row and column block, max and sum of exp (wide output layers)
    EPI_DZT = 6,   // logits recomputed with the roles of the operands exchanged (rows = classes, columns = samples):
                   // store dz^T[n][b] = (exp(z[b][n] - lse[b]) - [n == y_b]) / B in the storage dtype.  A tile of
                   // dz^T is one contiguous piece of memory; a tile of dz [b][n] would be 128 pieces 2 N_t bytes apart
    EPI_UPDATE_ACC = 7   // EPI_UPDATE whose accumulators start at -w / lr (chosen by the launcher, not by callers)
};

// C[g][m][n] (+)= sum_k A_g(m,k) * B_g(n,k), element (m,k) of A at A + g*gA + m*sam + k*sak.
struct GemmArgs {
    const void *A; int64_t sam, sak, gA;
    const void *B; int64_t sbn, sbk, gB;
    void *C; int64_t ldc, gC;
    int32_t M, N, K, G;
    const void *bias; int64_t gBias;          // EPI_FWD_*: bias[n] (may be null)
    const void *mask; int64_t ldm, gMask;     // EPI_BWD_DATA: keep where mask[m][n] > 0
    float lr;                                 // EPI_UPDATE: C = C - lr * acc
    float alpha = 1.0f;                       // forward: alpha * acc + bias; backward-data: alpha * acc (layer factor)
    float *partial; size_t partial_bytes;     // split-K scratch (fp32 partial products), may be null
    int32_t keep_partial;                     // host flag: a k-split launch leaves the partial products unfinished
    const void *zeros;                        // >= 16 bytes of zeros, 16-byte aligned (MFMA kernels)
    // EPI_LSE / EPI_DZT (softmax cross-entropy over a wide output layer, logits never stored)
    const int32_t *y; int64_t gY;             // labels of the batch rows, per-group stride
    float *pmax, *psum; int32_t nb;           // [G][M][nb] per column block: max, sum exp(z - max)
    float *zlabel;                            // [G][M] logit of the label
    const float *lse;                         // EPI_DZT: [G][N] log-sum-exp of the sample (a column there; y likewise)
    float invB;
    // EPI_DZT reuses pmax / nb (optional, pmax may be null): pmax[(g * nb + blk) * M + m] = sum over the samples of
    // column block blk (as wide as a wave tile) of the stored dz^T[m][.] - the bias gradient in nb partials per class,
    // added up in order by the bias kernel.  (A separate pair of fields would lengthen the argument block of every
    // instantiation; the row-statistics kernel was measured 13 % slower with it.)
};
// column-block width (elements) the EPI_LSE epilogue reduces over, for this problem shape
int lse_block_width(int dtype, int32_t M, int32_t N, int32_t K, int32_t G);
// the same for the sample (column) blocks of the EPI_DZT launch of this shape (M = classes, N = samples)
int dzt_block_width(int dtype, int32_t M, int32_t N, int32_t K, int32_t G);
hipError_t launch_lse_combine(const float *pmax, const float *psum, int32_t nb, float *qmax, float *qsum,
                              const float *zlabel, const int32_t *y, int64_t gY, int64_t Cn, float *lse,
                              float *rowloss, int32_t G, int32_t B, hipStream_t st);
constexpr int kLseChunksHost = 32;   // second-level partials per row (matches the kernels)
struct SplitPlan { int tile; int splits; int k_per_split; int kg; int64_t tiles; int cover; /* 1: one 256x128 block per group and split */ };
SplitPlan plan_gemm(int32_t M, int32_t N, int32_t K, int32_t G, bool allow_split, int esz);
hipError_t launch_gemm(int dtype, int epi, const GemmArgs &a, hipStream_t st);
// Number of k-splits launch_gemm uses for this product (1: none).  With a.keep_partial set, a split
// launch only writes a.partial, laid out [g * splits + sp][M][N] in fp32 without the bias, and the
// caller's next kernel adds the splits up; unsplit launches are not affected.
int gemm_splits(int dtype, int epi, const GemmArgs &a);
// The EPI_UPDATE products of several layers (independent of each other); small ones share one launch.
// gemm_update_shares_launch tells which do (the others are better launched, and timed, one by one).
bool gemm_update_shares_launch(int dtype, const GemmArgs &a);

hipError_t launch_splitk_finish_bwd(int dtype, const GemmArgs &a, const float *partial, int splits, hipStream_t st);

// ---- wide output layer, bf16, at most 128 hidden neurons per subnet and 256 samples: the last layer's part of a
// local step in two persistent launches that keep the hidden activations in LDS and stream the class tiles of W_t.
struct WideOutArgs {
    const void *h; int64_t ldh, gH;          // h_{t-1} [G][B][ldh] in bf16
    void *W; int64_t gW;                     // W_t blocks [G][N][C], updated in place by the backward launch
    void *bias; int64_t gBias;               // b_t [G][N] or null, updated in place by the backward launch
    const int32_t *y; int64_t gY;            // labels [G][B] (stride gY between groups)
    int32_t G, B, C; int64_t N;              // subnets, samples, hidden width per subnet, classes
    float alpha, lr_w, lr_b, invB;           // logits factor, step of the weights (lr * factor), step of the bias
    float *pmax, *psum; int32_t nb;          // statistics launch: per (group, workgroup, sample) max and sum exp
    float *zlabel;                           // statistics launch: logit of the label [G][B]
    const float *lse;                        // backward launch: log-sum-exp per sample [G][B]
    float *partial;                          // backward launch: dh partial sums [G * nb][B][C] fp32
    const void *zeros;                       // 256 zero bytes: what a request outside the matrices reads
};
bool wide_out_supported(int dtype, int32_t B, int64_t C, int64_t N);
int wide_out_workgroups(int32_t G);          // workgroups per subnet (= nb, = the number of dh partials)
hipError_t launch_wide_out_stats(const WideOutArgs &a, hipStream_t st);
hipError_t launch_wide_out_backward(const WideOutArgs &a, hipStream_t st);

hipError_t launch_softmax_xent(const float *logits, const int32_t *y, int64_t y_stride_g,
                               void *dz, float *rowloss, int32_t G, int32_t B, int64_t Cn,
                               int64_t ld, int dtype, hipStream_t st);
// The same for at most kXentRowsMaxC classes, reading either stored logits (splits == 1, bias == null)
// or the partial products of a k-split forward product (element strides between splits / groups / rows).
constexpr int kXentRowsMaxC = 256;
hipError_t launch_xent_rows(const float *z, int32_t splits, int64_t split_stride, int64_t g_stride, int64_t ldz,
                            const void *bias, int64_t gBias, const int32_t *y, int64_t y_stride_g, void *dz,
                            int64_t ld, float *rowloss, int32_t G, int32_t B, int32_t Cn, int dtype, hipStream_t st,
                            float alpha = 1.0f /* factor of the summed partial products, before the bias */);
// row losses of up to this many steps wait in the workspace for one reduction launch
constexpr int kLossSlots = 16;
// Section 2.2 standardisation of hidden-neuron inputs over the mini-batch, per subnet g and column r:
// forward: zh = (z - mean_b z) / sqrt(var_b z + eps) -> dtype, h = max(zh, 0), isg = 1 / sigma;
// backward (in place on dz, which holds dzh = dh * [zh > 0]):
//   dz = (dzh - mean_b dzh - zh * mean_b(dzh * zh)) * isg.
hipError_t launch_norm_forward(const float *z, void *zh, void *h, float *isg, int32_t G, int32_t B, int64_t R,
                               int64_t ld, float eps, int dtype, hipStream_t st);
hipError_t launch_norm_backward(void *dz, const void *zh, const float *isg, int32_t G, int32_t B, int64_t R,
                                int64_t ld, int dtype, hipStream_t st);
// loss_out[g * out_stride_g + j] = mean_b rowloss[j][g][b], j < nsteps
hipError_t launch_loss_reduce(const float *rowloss, float *loss_out, int64_t out_stride_g,
                              int32_t G, int32_t B, int32_t nsteps, hipStream_t st);
// bias[g][r] -= lr * sum_{blk < nrb} rsum[(g * nrb + blk) * R + r], blocks added in ascending order
hipError_t launch_bias_apply(void *bias, const float *rsum, int32_t nrb, int64_t R, int32_t G, float lr, int dtype,
                             hipStream_t st);
struct BiasJob { void *bias; const void *dz; int64_t R, ld; int32_t blk0; };
constexpr int kMaxBiasJobs = 16;
struct BiasArgs { BiasJob job[kMaxBiasJobs]; int32_t njobs, B, G; float lr; };
hipError_t launch_bias_update(BiasArgs &a, int dtype, hipStream_t st);
// true if every job of `a` takes the narrow kernel (so that the jobs can ride along with another launch)
bool bias_jobs_all_narrow(const BiasArgs &a, int dtype);
// `bias` (optional): narrow bias updates of the same step; *bias_done = they were done inside the shared launch
hipError_t launch_gemm_updates(int dtype, const GemmArgs *args, int n, const BiasArgs *bias, bool *bias_done,
                               hipStream_t st);

// sparse-input first layer (weights stored [G][N0][w])
struct CsrArgs {
    const int32_t *rowptr, *colidx; const void *vals; int64_t nnz;
    int64_t row0, stride_g;   // sample b of group g is CSR row row0 + g*stride_g + b
    int32_t G, B; int64_t N0, w;
    int64_t ld;               // row pitch of h_1 / dz_1
    float alpha = 1.0f;       // forward: alpha * (x W^T) + bias (layer factor)
};
// z_out != null: write the fp32 pre-activation there instead of ReLU(.) to h
// zero fill by a kernel (safe to record into a HIP graph); bytes is rounded down to a multiple of 4
hipError_t launch_fill_zero(void *p, size_t bytes, hipStream_t st);
// n 32-bit words set to v, by a kernel as well
hipError_t launch_fill_u32(void *p, int64_t n, uint32_t v, hipStream_t st);
// rowmajor: Wt is W_1 itself, [w][N0] (full-network evaluation), not the transposed subnet block
hipError_t launch_csr_forward(const CsrArgs &c, const void *Wt, const void *bias, void *h, float *z_out,
                              int dtype, hipStream_t st, bool rowmajor = false);
// bitmap: scratch of csr_scratch_bytes(G, N0, B) bytes, 8-byte aligned (cleared by the call itself)
size_t csr_scratch_bytes(int64_t G, int64_t N0, int64_t B);
hipError_t launch_csr_update(const CsrArgs &c, void *Wt, const void *dz, uint32_t *bitmap,
                             float lr, int dtype, hipStream_t st);

}  // namespace ist
