/*
 * sconv -- direct sparse convolution on MI355X (gfx950), C ABI.
 *
 * The operation (Section 2.1, Eq. (1) and Figure 2 of "Faster CNNs with Direct
 * Sparse Convolutions and Guided Pruning"; batch, stride, zero padding and
 * groups added):
 *
 *   out[n,k,y,x] = sum over the stored nonzeros j of CSR row k of
 *                  value[j] * in_pad[n, off[j] + y*stride*Wp + x*stride]
 *
 * The pruned weights of a layer are a CSR matrix with one row per output
 * channel k and one column per (c, r, s), c being the input channel inside the
 * row's group.  Each column index is lowered once, on the host, to the offset
 * off = ((g*Cg + c)*Hp + r)*Wp + s of element (c, r, s) in the zero-padded CHW
 * image (Hp = H + 2*pad, Wp = W + 2*pad, g = k / (K/groups), Cg = C/groups).
 * No im2col buffer and no dense weight matrix is ever formed.
 *
 * All functions return 0 (SCONV_OK) or a negative sconv_status; they never
 * throw.  Apart from a mutex-guarded record of which kernels have been enabled
 * for large LDS on which device, all state lives in the handles: distinct
 * handles may be used from distinct threads.  Pointers marked [host] are read or written on the CPU during the
 * call; pointers marked [device] are HIP device addresses that must stay valid
 * until the stream work enqueued by the call has finished.
 */
#ifndef SCONV_H
#define SCONV_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SCONV_OK = 0,
    SCONV_ERR_NULL = -1,        /* a required pointer is NULL */
    SCONV_ERR_DESC = -2,        /* non-positive size, groups not dividing C or K, output smaller than 1x1 */
    SCONV_ERR_CSR = -3,         /* rowptr not starting at 0 / not monotone, column out of range or not strictly ascending */
    SCONV_ERR_BATCH = -4,       /* N < 1; sconv_fc_forward: N not a multiple of 4 (per tile of 1024) */
    SCONV_ERR_CAPACITY = -5,    /* caller's buffer too small (export) */
    SCONV_ERR_PLAN = -6,        /* a tiling the kernels cannot run was requested */
    SCONV_ERR_HIP = -7,         /* a HIP call failed; sconv_last_hip_error() has its code */
    SCONV_ERR_NOMEM = -8,       /* host allocation failed */
    SCONV_ERR_RANGE = -9        /* sizes overflow 32-bit offsets inside one image */
} sconv_status;

/* Layer geometry (Section 2.1's problem statement).  The batch size is per call. */
typedef struct {
    int32_t C, H, W;            /* input channels, height, width (unpadded) */
    int32_t K, R, S;            /* output channels (filters), filter height, width */
    int32_t stride, pad, groups;
} sconv_desc;

/*
 * How the kernels tile a layer.  Zero in every field asks the library to choose.
 * kernel: 1 = LDS-tiled kernel with one nonzero stream per row (stride 1),
 * 3 = LDS-tiled kernel with one stream per wave (stride 1, nt = 4), two block
 * buffers in LDS and a barrier per channel block,
 * 4 = the same kernel with three block buffers and no barriers: the waves of a
 * workgroup tell each other through counters in LDS which blocks have landed
 * and drift up to half a block apart instead of all waiting for the slowest at
 * every block (takes everything kernel 3 takes: strips, splits, bands),
 * 2 = direct kernel (any stride).
 * For the LDS-tiled kernels one workgroup owns `nt` images (1, or a multiple of
 * 4), a band of `band` consecutive output rows (0 = choose; OH = the whole
 * image) and `waves/cg * rows_w` CSR rows; it walks the input channels in
 * blocks of `cb`; each wave keeps rows_w x t x (4 if nt >= 4 else 1)
 * accumulators per lane.  `strip` (kernels 3 and 4 only): 0 = the lanes of a wave
 * span 64 consecutive cells of the padded plane, chunk after chunk; w > 0 =
 * they span a block of 64/w output rows by w output columns and the t chunks of
 * a wave are t such blocks side by side (t*w >= OW, band <= cg * (64/w)),
 * which wastes fewer lanes when OW is a little under t*w.  `splits` (kernels 3
 * and 4 only; 0 or 1 = none): that many workgroups share the channel blocks of a
 * tile, for launches that would otherwise leave compute units idle; each
 * stores its partial results into scratch memory the handle owns and a second
 * launch adds them up in a fixed order.
 */
typedef struct {
    int32_t kernel, nt, cb, waves, cg, rows_w, t, band, strip, splits;
} sconv_plan;

typedef struct sconv_csr sconv_csr; /* opaque, owned by the library */

/*
 * Compress pruned dense weights [host] laid out [K][C/groups][R][S] into CSR,
 * lower the column indices to offsets, and pack for the kernels.  Entries equal
 * to zero (either sign) are dropped; every other value (denormal, NaN, Inf) is
 * kept.  Host work only: device copies are made by the first sconv_forward.
 * `plan` may be NULL.  On success *out receives a handle to free with
 * sconv_destroy_csr.
 */
int sconv_create_csr(const sconv_desc *desc, const float *dense_w, const sconv_plan *plan, sconv_csr **out);

/*
 * Same, from caller-built CSR arrays [host] (Figure 2's rowptr / colidx /
 * value): rowptr[K+1] with rowptr[0] == 0, colidx[nnz] in [0, (C/groups)*R*S)
 * strictly ascending inside each row and equal to (c*R + r)*S + s, values[nnz]
 * kept exactly as given (explicit zeros included).  The arrays are copied.
 */
int sconv_create_csr_from_arrays(const sconv_desc *desc, const int32_t *rowptr, const int32_t *colidx,
                                 const float *values, const sconv_plan *plan, sconv_csr **out);

/*
 * The lowering step alone, for either of two layouts of the zero-padded input
 * image (Section 2.1: the method needs only a layout function f with
 * f(c, y+r, x+s) = f(c, y, x) + f(0, r, s)):
 *   SCONV_LAYOUT_CHW  f(c,y,x) = (c*Hp + y)*Wp + x   (Figure 2's example; what the kernels read)
 *   SCONV_LAYOUT_HWC  f(c,y,x) = (y*Wp + x)*C + c    (channel innermost)
 * rowptr / colidx [host] as for sconv_create_csr_from_arrays; off[nnz] [host]
 * receives f(g*Cg + c, r, s) per nonzero, in CSR order.  *step_y and *step_x
 * (may be NULL) receive f(0, stride, 0) and f(0, 0, stride): output (y, x) reads
 * in_pad[off + y * step_y + x * step_x].  Host arithmetic only.  The device
 * entry points take CHW inputs; an HWC tensor has to be run through a loop of
 * the caller's own, which is what this function prepares.  SCONV_ERR_DESC for
 * an unknown layout.
 */
typedef enum { SCONV_LAYOUT_CHW = 0, SCONV_LAYOUT_HWC = 1 } sconv_layout;
int sconv_lower_offsets(const sconv_desc *desc, int32_t layout, const int32_t *rowptr, const int32_t *colidx,
                        int32_t *off, int32_t *step_y, int32_t *step_x);

/* Sizes and the tiling in use.  Any output pointer may be NULL. */
int sconv_csr_info(const sconv_csr *h, int64_t *nnz, int32_t *out_h, int32_t *out_w, sconv_plan *plan);

/*
 * Canonical lowered CSR (Figure 2's arrays after lowering): rowptr[K+1],
 * off[nnz] ascending in each row, values[nnz], all [host], caller-allocated.
 * *nnz_io holds the capacity of off/values on entry and the count on return
 * (SCONV_ERR_CAPACITY if too small; the count is still returned).
 */
int sconv_csr_export(const sconv_csr *h, int32_t *rowptr, int32_t *off, float *values, int64_t *nnz_io);

/*
 * Undo the kernel packing: walks the packed (reordered, channel-blocked,
 * byte-offset) arrays the kernels read and rebuilds canonical lowered CSR from
 * them alone.  `which` = 1 for the LDS-tiled kernel's arrays (SCONV_ERR_PLAN if
 * the handle has none), 2 for the direct kernel's, 3 for the arrays
 * sconv_fc_forward last packed (SCONV_ERR_PLAN before its first plan).  Same conventions as
 * sconv_csr_export.  Equality of the two exports shows the packing loses and
 * invents nothing.
 */
int sconv_csr_unpack(const sconv_csr *h, int32_t which, int32_t *rowptr, int32_t *off, float *values, int64_t *nnz_io);

/*
 * out[N][K][OH][OW] = sparse convolution of in[N][C][H][W], both [device],
 * contiguous fp32; `in` is NOT padded (padding is applied on chip).  `out` is
 * overwritten, rows without nonzeros with zeros.  Enqueued on `hip_stream`
 * (a hipStream_t; NULL = the default stream) of the current device and not
 * waited for.  `in` and `out` must not overlap.  A tiling the library chose
 * itself follows N: the first call with a new batch size chooses and packs for
 * it (host work, milliseconds, then a device allocation and a blocking upload:
 * that call synchronises with the device); the packings of the last four
 * tilings stay on the device, so alternating batch sizes cost nothing more.
 * If packing for a new N fails the handle keeps the packing it had.
 * Calls on one handle must not overlap in time (the handle owns scratch);
 * different handles are independent.
 */
int sconv_forward(sconv_csr *h, const float *in, float *out, int32_t N, void *hip_stream);

/*
 * sconv_forward for callers that cannot allocate device memory: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same kernels, same result bit for bit.  What sconv_forward keeps in
 * scratch memory it allocates and grows (the partial results of tilings that
 * split the input channels over workgroups, the phase images of strided
 * layers) lives here in a static device array of SCONV_NOALLOC_SCRATCH_BYTES
 * that the library's code object carries (each GPU the library runs on holds
 * it until the process ends).  The call allocates and frees nothing, on the
 * device or through any library, and never re-plans or uploads: the handle
 * must already hold, on the device, the packing for this N (one earlier
 * sconv_forward, sconv_forward_fused or sconv_tune call with the same N on this
 * device does that; the packings of the last four tilings stay resident).
 * SCONV_ERR_PLAN if it does not, or if the handle runs another kernel than the
 * flat-stream one; SCONV_ERR_CAPACITY if this layer and N need more scratch
 * than the array holds.  Nothing in the array has to start at zero (every
 * byte that is read is written first by the same call).  Every call on a GPU
 * shares that GPU's array: calls that overlap in time on one GPU race, also
 * on different handles and streams.
 */
#define SCONV_NOALLOC_SCRATCH_BYTES (64u << 20)
int sconv_forward_noalloc(sconv_csr *h, const float *in, float *out, int32_t N, void *hip_stream);

/*
 * The same with a bias and a ReLU applied before the result is stored: out =
 * max(conv + bias[k], 0).  Not part of the paper's method: the networks it
 * evaluates (Section 3) apply both after every convolution, and fusing them
 * saves a pass over the output.  `bias` [device] holds K
 * floats or is NULL (none); relu != 0 clamps at zero.  The flat-stream kernel
 * applies both to its accumulators; the other kernels run an elementwise pass
 * of their own after the convolution, and launches that split the channels
 * over workgroups apply them while adding up the partial results.
 */
int sconv_forward_fused(sconv_csr *h, const float *in, float *out, int32_t N, const float *bias, int32_t relu,
                        void *hip_stream);

/* The last HIP error code seen by a call on this handle (0 if none). */
int sconv_last_hip_error(const sconv_csr *h);

void sconv_destroy_csr(sconv_csr *h);

const char *sconv_strerror(int status);

/* ---- fully connected layers as sparse x dense matrix products (end of Section 2.1) ---- */

/*
 * out_t[K][N] = W x in_t[C][N]: W is the CSR matrix of a handle created for a
 * layer with H = W = R = S = 1, stride 1, pad 0, groups 1 (weights [K][C];
 * SCONV_ERR_DESC otherwise), the activations are feature-major, both [device],
 * contiguous fp32, one row of N images per feature.  N must be a multiple of
 * 4, and of 4 * ceil(N / 1024) above 1024 (SCONV_ERR_BATCH).  `bias` [device,
 * K floats] may be NULL; relu != 0 clamps at zero.  The same kernel as the
 * convolution's runs it: a feature's row is a channel plane, four consecutive
 * images one cell, the rows of W are register-blocked per wave and the features
 * walked in blocks staged through LDS, shared by several workgroups when K
 * alone gives too few (`splits` of the plan).  The arrays are packed for N on
 * the first call with that N.  `out_t` is overwritten; enqueued on `hip_stream`.
 * Any 4-byte-aligned `in_t` is accepted; one that is 16-byte aligned is staged
 * a cell (16 bytes) per lane instead of a float per lane, which is faster and
 * gives the same sums bit for bit.
 */
int sconv_fc_forward(sconv_csr *h, const float *in_t, float *out_t, int32_t N, const float *bias, int32_t relu,
                     void *hip_stream);

/* The tiling sconv_fc_forward uses for batch N (packs for it if it has not yet). */
int sconv_fc_plan(sconv_csr *h, int32_t N, sconv_plan *plan);

/* ---- measured choice of the tiling -------------------------------------------- */

/*
 * The tiling of a layer (channel block, workgroup size, rows per wave, bands,
 * strips, channel splits) is chosen by a cost model (the blocking parameters
 * Section 2.1 leaves to tuning).  sconv_tune runs the `max_plans` tilings the
 * model ranks best for batch size N (1..32; <= 0 means 8) on the caller's
 * buffers, timing each with events on `hip_stream`, and keeps the fastest (the
 * model's own choice unless another is at least 1.5 % faster) for later
 * sconv_forward / sconv_forward_fused calls with this N.  `in` and `out`
 * [device] are as for sconv_forward; on return `out` holds the layer's output.
 * SCONV_ERR_PLAN when the handle was created with a tiling of the caller's or
 * has no LDS path.  It packs, allocates, uploads and waits for the stream, so it
 * belongs to set-up, not to a captured or latency-critical region.  The same
 * rules as for sconv_forward apply to overlapping calls on one handle.
 */
int sconv_tune(sconv_csr *h, const float *in, float *out, int32_t N, int32_t max_plans, void *hip_stream);

/*
 * The candidates sconv_tune would time for batch size N, best-ranked first:
 * plans[0] is the cost model's choice, the one sconv_forward uses untuned.
 * `plans` [host] has room for max_plans entries (1..32; <= 0 means 8); *count
 * receives how many were written.  Every one of them is a complete tiling that
 * sconv_create_csr accepts for this layer.  No GPU is needed.
 */
int sconv_rank_plans(const sconv_csr *h, int32_t N, int32_t max_plans, sconv_plan *plans, int32_t *count);

/* The same for sconv_fc_forward (no bias, no ReLU while timing; the choice holds for calls with either). */
int sconv_fc_tune(sconv_csr *h, const float *in_t, float *out_t, int32_t N, int32_t max_plans, void *hip_stream);

/* ---- roofline performance model (Section 2.2) ------------------------------ */

/*
 * Machine parameters.  dense_flops (F) and hbm_bytes_per_s (B) are ACHIEVABLE
 * rates, as the paper takes them from SGEMM and STREAM.  alpha > 0 is used as
 * given (the paper's form); alpha <= 0 derives it from the ceilings of the
 * sparse kernel:
 *   F_sparse = lane_efficiency * min(fma_flops, 2 * lds_bytes_per_s / lds_bytes_per_fma)
 *   alpha    = dense_flops / F_sparse
 */
typedef struct {
    double dense_flops;       /* F, FLOP/s of dense convolution (GEMM proxy) */
    double hbm_bytes_per_s;   /* B */
    double alpha;             /* compute overhead of the sparse kernel, or <= 0 */
    double beta;              /* storage overhead of CSR: 2 (4 B index per 4 B value) */
    double fma_flops;         /* FP32 multiply-add ceiling of the sparse kernel, FLOP/s */
    double lds_bytes_per_s;   /* LDS read bandwidth, whole chip */
    double lds_bytes_per_fma; /* LDS bytes read per multiply-add (4: one fp32 operand) */
    double lane_efficiency;   /* fraction of that ceiling the kernel sustains as useful multiply-adds
                                 (lanes that are real outputs x issue slots not lost to address
                                 arithmetic, waits and barriers) */
    double t_fixed;           /* seconds per call outside the paper's model (launch, prologue, first
                                 block, last stores), added to the sparse time; 0 = the formulas as
                                 Section 2.2 prints them */
} sconv_machine;

typedef struct {
    double flops_dense;       /* C: 2*K*Cg*R*S*OH*OW*N */
    double bytes_act;         /* S_A: 4*N*(C*H*W + K*OH*OW) */
    double bytes_w;           /* S_W: 4*K*Cg*R*S */
    double density;           /* x used (the handle's realised density if one was given) */
    double alpha;             /* alpha used */
    double t_dense;           /* C/F, seconds */
    double t_sparse_compute;  /* alpha*x*C/F */
    double t_sparse_bw;       /* (S_A + beta*x*S_W)/B */
    double t_sparse;          /* max of the two (+ the machine's t_fixed) */
    double speedup;           /* t_dense / t_sparse */
    double effective_flops;   /* C / t_sparse (zeros counted) */
    double actual_flops;      /* x*C / t_sparse (nonzeros only) */
    double x_upper;           /* density where t_sparse_compute == t_sparse_bw (inf if never) */
    double x_lower;           /* 1/alpha: above it sparse is slower than dense */
    int32_t bandwidth_bound;  /* 1 if t_sparse_bw > t_sparse_compute */
} sconv_prediction;

/* Measured defaults for one MI355X (t_fixed included: set it to 0 for the paper's formulas alone). */
void sconv_machine_gfx950(sconv_machine *m);

/*
 * Evaluate the model for a layer at batch N and density x.  If `h` is not NULL
 * its realised density nnz/(K*Cg*R*S) replaces `density`.  `m` NULL = the
 * gfx950 defaults.  Pure host arithmetic.
 */
int sconv_model_predict(const sconv_desc *desc, int32_t N, double density, const sconv_csr *h,
                        const sconv_machine *m, sconv_prediction *out);

/*
 * The same model for sparse convolution on LOWERED tensors, the curve the
 * figure of Section 2.2 draws beside the direct one: lowering replicates the
 * input (Section 2.1), so S_A becomes 4*N*(C*R*S*OH*OW + K*OH*OW), the lowered
 * matrix plus the output; everything else is unchanged.  The cost of creating
 * the lowered matrix is not charged.  Only the model: no lowering-based kernel
 * is part of this library.
 */
int sconv_model_predict_lowered(const sconv_desc *desc, int32_t N, double density, const sconv_csr *h,
                                const sconv_machine *m, sconv_prediction *out);

/*
 * How evenly the packing spreads the nonzeros (the load-balance step of the
 * path; the paper only asks that all cores be used, Section 3).  The waves of a
 * workgroup meet at a barrier after every channel block, so a block costs what
 * its longest wave stream costs.  All counts are in stream chunks of 8 entries
 * (a segment may open with a half chunk of 4).
 * Only for handles packed for kernel 3 (SCONV_ERR_PLAN otherwise).
 */
typedef struct {
    int64_t nnz;             /* real nonzeros */
    int64_t stream_entries;  /* entries in the streams, chunk padding included */
    double wave_mean;        /* sum over (workgroup, block) of the mean stream length of its waves */
    double wave_max;         /* same with the longest wave: wave_max / wave_mean >= 1 is the barrier loss */
    double simd_max;         /* same with the longest of the 4 SIMDs (waves w, w+4, ... summed, per wave) */
    double workgroup_mean;   /* mean over workgroups of their total of per-block longest streams */
    double workgroup_max;    /* the largest such total: the workgroup the launch waits for */
} sconv_balance;
int sconv_csr_balance(const sconv_csr *h, sconv_balance *out);

/* ---- the pruning controller's decision (Section 2.3, the Guided Sparsity Learning algorithm) ---- */

/*
 * What the algorithm does with one layer, given the model.  The algorithm's two
 * sparsity bounds are stated as densities here: x_upper is the density below
 * which the layer is bandwidth bound and pruning brings no more speed (the
 * algorithm's upper sparsity bound); x_lower = 1/alpha is the density above
 * which the sparse kernel is slower than dense convolution (its lower sparsity
 * bound).
 */
typedef enum {
    SCONV_GSL_EXCLUDE = 0,        /* no useful range (x_upper >= x_lower): never prune this layer */
    SCONV_GSL_PRUNE = 1,          /* inside or above the useful range and still moving: keep pruning */
    SCONV_GSL_STOP = 2,           /* density <= x_upper: stop pruning, the other layers get the room */
    SCONV_GSL_RESTORE_DENSE = 3   /* density has stabilised at or above x_lower: stop and restore the dense weights */
} sconv_gsl_action;

/*
 * Decide for one layer at batch N with current nonzero density `density`
 * (in (0, 1]); `stabilized` != 0 says the density has stopped changing.  `m`
 * NULL = the gfx950 defaults.  *pred (may be NULL) receives the model's
 * prediction the decision was taken on.  Pure host arithmetic; only the
 * decision is built here, not the training loop around it.
 */
int sconv_gsl_decide(const sconv_desc *desc, int32_t N, double density, int32_t stabilized, const sconv_machine *m,
                     int32_t *action, sconv_prediction *pred);

#ifdef __cplusplus
}
#endif
#endif /* SCONV_H */
