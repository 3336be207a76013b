/*
 * ist.h - C ABI of the MI355X (gfx950) hot path of Independent Subnet Training.
 *
 * Paper: "Distributed Learning of Fully Connected Neural Networks using
 * Independent Subnet Training" (IST).  One IST round is
 *
 *     ist_partition  ->  ist_subnet_steps (k local SGD steps)  ->  ist_merge
 *
 * with all S subnets resident on one GPU.  Notation follows the paper: layers
 * 0..t, N_l neurons at layer l, W_l in R^{N_l x N_{l-1}} with f_l = W_l f_{l-1}
 * (Appendix A), S = the paper's n sites, k = the paper's J local iterations.
 *
 * Conventions
 *   - Every pointer marked [device] is GPU memory owned by the caller (for
 *     instance a PyTorch tensor); the library never allocates or frees device
 *     memory.  Pointers marked [host] are ordinary host memory read during the
 *     call only.  Structs themselves are host memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls enqueue work on it and return; results are ready when the stream
 *     reaches that point.
 *   - All functions return an ist_status (0 = IST_OK, < 0 = error), never throw
 *     and never abort.  Argument errors are detected on the host before anything
 *     is enqueued.  ist_last_error() gives a text for the last failure.
 *   - Matrices are row-major.  Storage types: IST_F32 (IEEE binary32) or
 *     IST_BF16 (bfloat16); accumulation is always binary32.
 */
#ifndef IST_H
#define IST_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    IST_OK = 0,
    IST_EINVAL = -1,       /* null pointer, non-positive size, bad enum */
    IST_ESHAPE = -2,       /* a hidden layer narrower than S, B > max_B, ... */
    IST_EPERM = -3,        /* a perm is not a permutation of 0..N_l-1 (checked mode) */
    IST_ENOMEM = -4,       /* a bound buffer is too small */
    IST_EHIP = -5,         /* a HIP runtime call failed */
    IST_ESTATE = -6,       /* call order violated (steps/merge before partition, no bind) */
    IST_EUNSUPPORTED = -7  /* valid request the library does not implement */
} ist_status;

typedef enum { IST_F32 = 0, IST_BF16 = 1 } ist_dtype;
typedef enum { IST_DENSE = 0, IST_CSR = 1 } ist_input_kind;

/* The full network and how it is split. [host] */
typedef struct {
    int32_t t;             /* number of weight matrices, >= 2 (at least one hidden layer) */
    const int64_t *dims;   /* [host] N_0..N_t, t+1 entries; every hidden width N_1..N_{t-1} >= S */
    int32_t S;             /* number of subnets, >= 1 */
    int32_t dtype;         /* ist_dtype: storage of W, b, activations, inputs */
    int32_t input;         /* ist_input_kind of the mini-batches */
    int32_t has_bias;      /* 1: biases b_1..b_t exist, 0: none */
    int32_t normalize;     /* 1: Section 2.2 "Correcting Distributional Shift": every hidden neuron's input
                              is standardised over the mini-batch before the activation, z <- (z - mu) / sigma
                              with mu, sigma^2 the mean and (biased) variance over the B samples of the step,
                              sigma = sqrt(var + norm_eps); the gradient flows through mu and sigma.  0: plain
                              ReLU network. */
    float norm_eps;        /* > 0; values <= 0 select 1e-5 */
    const float *layer_scale; /* [host] t factors gamma_1..gamma_t (finite, > 0), or NULL for none.  Appendix A,
                              equation (4): the subnet's product of layer l is multiplied by gamma_l,
                              z_l = gamma_l (W_l f_{l-1}) + b_l, and so are the gradients that flow through it.
                              The paper's factor is n^2 = S^2 where both sides of W_l are partitioned (each
                              subnet's masked output is then an unbiased estimate of the full product);
                              Section 2.2 drops it in favour of `normalize`.  Read by ist_create only. */
} ist_model_desc;

/* Full parameters, caller-owned. [host struct, device arrays] */
typedef struct {
    void *const *W;        /* [host] t pointers; W[l-1] -> [device] row-major [N_l][N_{l-1}] */
    void *const *b;        /* [host] t pointers; b[l-1] -> [device] [N_l]; NULL if has_bias == 0 */
} ist_params;

/* Mini-batches for all S subnets and k steps: sample b of step j of subnet s is
 * row  s*stride_s + j*stride_k + b.  Every (s, j) normally has its own batch;
 * stride 0 reuses one.  [host struct, device arrays] */
typedef struct {
    const void *x;         /* dense: [device] rows of N_0 values in the model dtype */
    const int32_t *rowptr; /* CSR: [device] row offsets, (max row index + 2) entries */
    const int32_t *colidx; /* CSR: [device] column ids, ascending inside a row, < N_0 */
    const void *vals;      /* CSR: [device] values in the model dtype */
    int64_t nnz;           /* CSR: length of colidx / vals */
    const int32_t *y;      /* [device] class id per row, 0 <= y < N_t */
    int64_t stride_s;      /* rows between consecutive subnets */
    int64_t stride_k;      /* rows between consecutive steps */
    int32_t B;             /* mini-batch size, 1..max_B */
} ist_batch;

typedef struct ist_ctx ist_ctx;

/* Creates the host-side plan for one network shape.  No device work.
 * IST_ESHAPE if a hidden layer has fewer than S neurons or max_B < 1; IST_EUNSUPPORTED if S > 4096. */
ist_status ist_create(const ist_model_desc *desc, int32_t max_B, ist_ctx **out);
ist_status ist_destroy(ist_ctx *ctx);

/* Sizes of the two device buffers the caller must provide: `subnets` holds the
 * packed parameters of all S subnets plus the neuron index tables (private
 * layout), `workspace` holds activations, gradients and scratch for
 * ist_subnet_steps.  Both must be 256-byte aligned. */
ist_status ist_subnets_bytes(const ist_ctx *ctx, size_t *bytes);
ist_status ist_workspace_bytes(const ist_ctx *ctx, size_t *bytes);
ist_status ist_bind(ist_ctx *ctx, void *subnets /*[device]*/, size_t subnets_bytes,
                    void *workspace /*[device]*/, size_t workspace_bytes);

/* checked != 0: ist_partition synchronises the stream and returns IST_EPERM if a
 * permutation is invalid.  Unchecked (default), an invalid permutation gives
 * unspecified subnet contents but never an out-of-bounds access. */
ist_status ist_set_checked(ist_ctx *ctx, int32_t checked);

/*
 * ist_partition - Section 2.1 "Constructing Subnets", Appendix A.
 * perm[l-1] [device], l = 1..t-1, is a permutation of 0..N_l-1; subnet s owns
 * the s-th block H_l^s of perm_l, and all input and output neurons.  Blocks are as
 * equal as the width allows: with N_l = q S + r the first r subnets own q + 1
 * neurons and the others q, so H_l^s starts at position s q + min(s, r) (equal
 * blocks perm_l[s*N_l/S .. (s+1)*N_l/S - 1] when S divides N_l).  Copies W_l[H_l^s, H_{l-1}^s] and b_l[H_l^s]
 * into the bound subnet buffer for every s (bit-exact copies; the output bias
 * b_t is replicated).  `params` is only read.
 */
ist_status ist_partition(ist_ctx *ctx, const ist_params *params,
                         const int32_t *const *perm /*[host] t-1 [device] pointers*/,
                         void *stream);

/*
 * ist_subnet_steps - Section 2.1 "Training Subnets", Appendix B (local step
 * w <- w - lr * grad).  Runs k steps of mini-batch SGD on each of the S subnets
 * independently: forward through the narrow net (ReLU hidden units, no n^2
 * factor, Section 2.2), mean softmax cross-entropy, back-propagation, in-place
 * update of the subnet parameters.  Values are kept in the model dtype
 * (round-to-nearest-even): W, b, hidden activations and activation gradients;
 * logits, softmax, reductions and the update arithmetic are binary32.
 * loss_out: [device] float [S][k], mean loss of each step before its update,
 * or NULL.  May be called repeatedly between partition and merge.
 */
ist_status ist_subnet_steps(ist_ctx *ctx, const ist_batch *batch, float lr, int32_t k,
                            float *loss_out, void *stream);

/*
 * ist_merge - Section 2.1 "Training Subnets": subnet parameters are copied back
 * into the full network; blocks are disjoint so nothing collides, and entries
 * of W owned by no subnet keep their bits.  Hidden biases return to their
 * neuron; b_t becomes the mean over subnets (binary32 sum as a balanced pairwise
 * tree over the subnet index, times 1/S, rounded to dtype: exact for identical
 * copies when S is a power of two).  Writes `params` in place; subnets stay valid.
 */
ist_status ist_merge(ist_ctx *ctx, const ist_params *params, void *stream);

/*
 * Re-sampling between rounds (Section 2.1: subnets are re-sampled after every J local
 * iterations): exactly ist_merge(ctx, params) followed by ist_partition(ctx, params, perm)
 * - `params` ends up holding the merged network and the context the subnets of the new
 * permutation, bit for bit - but in one pass over each weight matrix: the row that merge
 * writes is the row partition would read back.  The new blocks are built in a second
 * subnet buffer given once with ist_bind_spare (same size and alignment as `subnets` of
 * ist_bind, caller-owned device memory, must stay valid while the context is used); the
 * two buffers change roles at every call (on the host: a HIP graph recorded from this call
 * keeps the roles it saw and must not be replayed; ist_partition, ist_subnet_steps and ist_merge
 * have no such state and may be); ist_bind forgets the spare (give it again after a
 * re-bind).  IST_ESTATE before ist_partition or without a
 * spare buffer; with checking on, a perm that is not a permutation gives IST_EPERM and
 * leaves `params` and the current subnets untouched.
 */
ist_status ist_bind_spare(ist_ctx *ctx, void *spare_subnets, size_t spare_bytes);
ist_status ist_resample(ist_ctx *ctx, const ist_params *params, const int32_t *const *perm, void *stream);

/*
 * ist_forward_full - the forward pass of the FULL network (every neuron of every layer, no
 * partition): logits = W_t f_{t-1} + b_t with f_l = ReLU(W_l f_{l-1} + b_l), the network of
 * Section 2.1 that the subnets are cut from and merged back into; with `normalize` set the
 * inputs of the hidden neurons are standardised with the statistics of this batch (Section 2.2:
 * after training, mu and sigma are computed with the full network over a subset of the data).
 * The full network has no masks, so layer_scale does not apply to it.
 * For evaluation between rounds.  Uses samples 0..B-1 of `batch` (x rows or CSR rows 0..B-1;
 * y and the strides are ignored), B <= max_B.  logits: [device] float [B][N_t].  Same storage
 * and accumulation types as ist_subnet_steps.  Needs ist_bind only; it overwrites the workspace
 * (not the subnets), so it must not run concurrently with ist_subnet_steps on another stream.
 */
ist_status ist_forward_full(ist_ctx *ctx, const ist_params *params, const ist_batch *batch,
                            float *logits /*[device]*/, void *stream);

/*
 * ist_forward_full_static - ist_forward_full for callers that cannot allocate device memory or hand
 * over a workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, same kernels and bit-identical logits, but it needs no ist_bind: the
 * hidden activations, the standardisation's intermediates and the split-k partial sums live in a
 * static device array of IST_STATIC_SCRATCH_BYTES inside the library (each GPU the library runs on
 * holds its own copy until the process ends).  The call allocates nothing and frees nothing; it
 * enqueues a clearing kernel for the part of the array it uses, then the pass itself.
 *   - IST_ENOMEM (with a text in ist_last_error) if this network and batch need more than the array
 *     holds: about B * sum of the hidden widths (rounded up to 8) * element size, plus B * width * 8
 *     bytes per hidden layer with `normalize`, plus the split-k scratch of the context.
 *   - Every call on a GPU uses that GPU's one array: calls that overlap in time on one GPU (different
 *     streams, or different contexts) race; callers serialise them.  It does not touch the bound
 *     workspace, so it may overlap ist_subnet_steps.
 *   - The first call on a device asks the runtime for the array's address; make that call once
 *     before a stream capture begins.  Profiling brackets (ist_profile_enable) are not recorded.
 */
#define IST_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
ist_status ist_forward_full_static(ist_ctx *ctx, const ist_params *params, const ist_batch *batch,
                                   float *logits /*[device]*/, void *stream);

/* Canonical view of one subnet's layer l (1..t) for inspection and tests:
 * dstW [device] row-major [rows][cols] with rows/cols in the order of the
 * permutation block (H_l^s order), dstb [device] [rows] or NULL. */
ist_status ist_subnet_export(ist_ctx *ctx, int32_t s, int32_t l, void *dstW, void *dstb,
                             void *stream);

/* Rows and columns of layer l of subnet s as ist_subnet_export writes them (ist_subnet_shape_of), and of
 * the widest subnet, which is subnet 0 (ist_subnet_shape; every subnet's when S divides the hidden widths). */
ist_status ist_subnet_shape(const ist_ctx *ctx, int32_t l, int64_t *rows, int64_t *cols);
ist_status ist_subnet_shape_of(const ist_ctx *ctx, int32_t s, int32_t l, int64_t *rows, int64_t *cols);

/*
 * Measurement support.  With profiling on, every kernel launch of the three hot
 * calls is bracketed by HIP events on the caller's stream (this perturbs timing
 * slightly; leave it off for throughput runs).  ist_profile_read synchronises
 * with the last recorded event and returns, for one kernel class, the summed
 * kernel time in milliseconds and the number of launches since the last reset.
 * Kernel classes are numbered 0 .. ist_profile_classes()-1.
 */
ist_status ist_profile_enable(ist_ctx *ctx, int32_t on);
ist_status ist_profile_reset(ist_ctx *ctx);
ist_status ist_profile_read(ist_ctx *ctx, int32_t kernel_class, double *total_ms, int64_t *launches);
int32_t ist_profile_classes(void);
const char *ist_profile_class_name(int32_t kernel_class);

/*
 * The same records grouped by kernel: one entry per distinct kernel label (kernel
 * and launch configuration, e.g. "gemm_fwd_relu_bf16_256x256_t512").
 * ist_profile_kernel_count returns the number of entries since the last reset;
 * ist_profile_kernel copies entry `index`: its label (NUL-terminated, truncated to
 * label_cap), its kernel class, the summed kernel time [ms], the number of launches,
 * and the algorithmic work summed over those launches: flops (2*M*N*K per product
 * and subnet; 0 for copy kernels) and bytes (products: every operand element read
 * once, every result written once, the weights of an update read and written, the
 * ReLU mask of a backward-data product read; copy kernels: the cache-line-granular
 * minimum - rows a block touches are read whole, and rewritten whole on merge when
 * their columns are partitioned; 0 where not tracked).  All pointers [host].
 */
ist_status ist_profile_kernel_count(ist_ctx *ctx, int32_t *count);
ist_status ist_profile_kernel(ist_ctx *ctx, int32_t index, char *label, size_t label_cap,
                              int32_t *kernel_class, double *total_ms, int64_t *launches,
                              double *flops, double *bytes);

const char *ist_last_error(const ist_ctx *ctx);
const char *ist_version(void);

#ifdef __cplusplus
}
#endif
#endif /* IST_H */
