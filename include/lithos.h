/*
 * liblithos - kernel atomization and CU-partition scheduling on one MI355X.
 *
 * C ABI.  Every call returns LITHOS_OK (0) or a negative LITHOS_E* code and
 * never throws; lithos_last_error() returns a thread-local text for the last
 * failure on the calling thread.
 *
 * Memory: the library never allocates, frees or copies tensor memory.  All
 * pointers inside lithos_op_t are DEVICE pointers owned by the caller, who
 * keeps them alive until the operation's completion has been observed.
 * Pointers in the call signatures themselves (out-parameters, masks, result
 * arrays) are HOST pointers unless a comment says "device".
 *
 * Method: LithOS (arXiv 2504.15465).  Citations below name its sections.
 */
#ifndef LITHOS_H
#define LITHOS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LITHOS_OK       0
#define LITHOS_EINVAL  -1   /* bad shape, alignment, flag or handle; nothing was launched */
#define LITHOS_EHIP    -2   /* a HIP call failed; text holds hipGetErrorString */
#define LITHOS_EMASK   -3   /* empty or out-of-range CU mask */
#define LITHOS_ESTATE  -4   /* call not valid in the object's current state */
#define LITHOS_ELIMIT  -5   /* a fixed capacity of the library was exceeded */

#define LITHOS_MASK_WORDS 8          /* 256 CUs = 8 x 32-bit words */
#define LITHOS_MAX_SWEEP  64         /* right-size sweep points */

typedef struct lithos_ctx lithos_ctx_t;
typedef struct lithos_partition lithos_partition_t;
typedef struct lithos_tenant lithos_tenant_t;

typedef struct { uint32_t x, y, z; } lithos_dim3;

/* ---- operators --------------------------------------------------------- */

enum {
    LITHOS_OP_GEMM      = 1,  /* C = op(A) op(B) [+bias][GELU][+residual], bf16 in, fp32 accumulate */
    LITHOS_OP_BIAS_ACT  = 2,  /* y = act(x + bias) */
    LITHOS_OP_LAYERNORM = 3,  /* per-row (x-mean)/sqrt(var+eps)*gamma+beta, biased variance */
    LITHOS_OP_SOFTMAX   = 4,  /* per-row softmax(scale * s) */
    LITHOS_OP_ATTN_ENC  = 5,  /* full (unmasked) multi-head attention on a packed qkv tensor */
    LITHOS_OP_ATTN_DEC  = 6,  /* one query token per sequence against a key/value cache, grouped-query */
    LITHOS_OP_RMSNORM   = 7,  /* x / sqrt(mean(x^2)+eps) * w */
    LITHOS_OP_ROPE_KV   = 8,  /* rotary embedding of q and k (rotate-half) + append k,v to the cache */
    LITHOS_OP_SILU_MUL  = 9,  /* silu(gate) * up on a packed [rows, 2F] tensor */
    LITHOS_OP_SPIN      = 10, /* test kernel: every block spins a fixed number of clock ticks */
    LITHOS_OP_ATTN_MERGE = 11, /* second step of a split ATTN_DEC: merges the key ranges' partial softmaxes */
    LITHOS_OP_SUM_SLICES = 12, /* second step of a K-sliced GEMM: adds the fp32 partial planes in slice order */
    LITHOS_OP_ATTN_PREFILL = 13 /* causal self-attention over a whole prompt (query i sees keys 0..i), grouped-query */
};

#define LITHOS_ATTN_MAX_SPLITS 64
#define LITHOS_GEMM_MAX_SLICES 64

/* flags (meaning depends on the kind, see the table below) */
#define LITHOS_F_TRANS_A   (1u << 0)   /* A is stored [K,M] */
#define LITHOS_F_TRANS_B   (1u << 1)   /* B is stored [N,K] */
#define LITHOS_F_BIAS      (1u << 2)   /* add bias[n] (fp32 vector) */
#define LITHOS_F_GELU      (1u << 3)   /* erf-form GELU after the bias */
#define LITHOS_F_RESIDUAL  (1u << 4)   /* add residual[m,n] (fp32) after the activation */
#define LITHOS_F_OUT_F32   (1u << 5)   /* out[0] is fp32 (default bf16) */
#define LITHOS_F_IN_F32    (1u << 6)   /* in[0] is fp32 (default bf16) */
#define LITHOS_F_SPLIT_A   (1u << 7)   /* GEMM: A is a bf16 pair hi + lo (two planes, dim[3] elements apart) */
#define LITHOS_F_OUT_SPLIT (1u << 8)   /* producer also writes the lo plane: lo = bf16(y - bf16(y)) */
#define LITHOS_F_NORM_LN   (1u << 9)   /* GEMM: rows of A pass through LAYERNORM (gamma in[4], column sums in[5], eps fparam0) on load */
#define LITHOS_F_NORM_RMS  (1u << 10)  /* GEMM: rows of A pass through RMSNORM (w in[4], eps fparam0) on load */
#define LITHOS_F_GLU       (1u << 11)  /* GEMM: B holds N gate rows then N up rows; C = silu(A gate^T) * (A up^T) */

/* GEMM tile selectors for lithos_op_t.tile (0 = library chooses) */
#define LITHOS_TILE_64     64    /* 64x64 output tile */
#define LITHOS_TILE_128    128   /* 128x128 */
#define LITHOS_TILE_256    256   /* 256x256 */
#define LITHOS_TILE_SKINNY 1     /* M <= 32 weight-streaming kernel; needs TRANS_B */

/*
 * One operator instance.  Unused fields are zero.
 *
 * kind        dim[]                              in[] / out[]                         ld[] / fparam[]
 * GEMM        M,N,K,[a_plane,c_plane,slices,     A,B,bias(f32),residual(f32),          lda,ldb,ldc,ldr
 *             slice_plane,colsum_stride]         [gamma(f32),colsums(f32)] / C         fparam0=eps (NORM_*)
 *             slices (dim[5]) > 1 cuts K into that many ranges of whole 64-wide k-tiles (balanced:
 *             range z holds the k-tiles [z*KT/S, (z+1)*KT/S)); the logical grid gets z = slices and
 *             block (x,y,z) writes its fp32 partial tile to plane z of out[0], dim[6] (>= M*ldc)
 *             elements after plane z-1.  Needs OUT_F32 and no epilogue flag; a wide K with few output
 *             tiles fills the chip that way.  SUM_SLICES on the same queue then adds the planes in
 *             slice order and applies the epilogue, so the result does not depend on how either
 *             launch was cut into atoms.
 *             NORM_LN / NORM_RMS and GLU fuse a decoder's or an MLP's row kernels into the weight-
 *             streaming form (TRANS_B, M <= 16; the NORM flags also need IN_F32).  C is the product of
 *             the rows that LAYERNORM / RMSNORM would have written in fp32, computed as
 *               r_m * (sum_k (x-c_m) gamma_k B_nk - (mean_m-c_m) * G_n) + H_n       (c_m = x[m,0]),
 *             RMSNORM: r_m * sum_k x gamma_k B_nk, so it differs from the two-step form by fp32 rounding
 *             only.  G_n = sum_k gamma_k B_nk and H_n = sum_k beta_k B_nk depend on the weights alone:
 *             the caller computes them once per weight matrix with this same GEMM (A = the two fp32 rows
 *             gamma and beta, IN_F32 | OUT_F32, same B) and passes the [2, dim[7]] result as in[5].
 *             GLU's C[m,n] is what SILU_MUL would have made of the [M,2N] product (B has 2N rows, and so
 *             have the column sums); it takes no BIAS, GELU, RESIDUAL or OUT_SPLIT.  Each saves a launch
 *             and the round trip of an intermediate tensor, which is what a request of a few rows is made of.
 * SUM_SLICES  rows,cols,slices,slice_plane       planes(f32),bias(f32),residual(f32) / y   ld0=row stride of the planes,
 *             y = act(sum_z plane_z + bias) + residual; BIAS, GELU, RESIDUAL, OUT_F32 as for GEMM          ld1=of y, ld2=of residual
 * BIAS_ACT    rows,cols                          x,bias(f32) / y
 * LAYERNORM   rows,H                             x,gamma(f32),beta(f32) / y,[y_bf16]   fparam0=eps
 * SOFTMAX     rows,n                             s / p                                fparam0=scale
 * ATTN_ENC    batch,heads,seq,d                  qkv[batch*seq,3*heads*d] / o[batch*seq,heads*d]  fparam0=scale
 * ATTN_DEC    batch,n_q,n_kv,d,keys,cap,splits   q,kcache,vcache,[workspace] / o      ld0=q row stride; fparam0=scale
 *             caches are [batch,cap,n_kv,d] bf16; the first `keys` positions are read.
 *             splits <= 1: one workgroup per (sequence, key/value head) writes o.
 *             splits > 1: the keys are cut into `splits` ranges, one workgroup each, which write
 *             partial softmaxes to the fp32 workspace in[3] (batch*n_q*splits*(d+2) floats) and
 *             leave o untouched; ATTN_MERGE on the same queue then produces o.
 * ATTN_MERGE  batch,n_q,n_kv,d,splits            workspace / o                        OUT_F32 as for ATTN_DEC
 * ATTN_PREFILL batch,n_q,n_kv,d,T,cap             q,kcache,vcache / o                  ld0=q row stride, ld1=o row stride;
 *             q [batch*T, ld0] and o [batch*T, ld1] bf16 with head h at columns h*d; the caches   fparam0=scale
 *             [batch,cap,n_kv,d] bf16 hold the prompt's T keys and values; d = 128, T a multiple of 256.
 *             One workgroup per (pair of 128-query tiles, sequence, query head): tile p from the end and
 *             tile p from the start of the prompt, so that every block sees T/128 + 1 tiles of keys; grid
 *             x = heads of a key/value head x pairs, y = key/value head, z = sequence.
 * RMSNORM     rows,H                             x,w(f32) / y                         fparam0=eps
 * ROPE_KV     rows,n_q,n_kv,d,pos,cap            qkv[rows,(n_q+2n_kv)d] (in place) / kcache,vcache   fparam0=theta
 *             qkv is bf16, or fp32 with IN_F32; the caches are always bf16 (rounded on append)
 * SILU_MUL    rows,F                             gu[rows,2F] / y[rows,F]
 * IN_F32 / OUT_F32 select fp32 for in[0] / out[0] of the row kernels and of ATTN_DEC's q / o;
 * GEMM takes IN_F32 (fp32 A) only in its M <= 32 weight-streaming form.
 * SPIN        blocks,ticks                       - / -
 *
 * Split bf16 ("hi + lo"): a tensor stored as two bf16 planes whose sum carries ~16 significant
 * bits.  GEMM reads A that way with SPLIT_A (MFMA tile kernels, 64 and 128 tiles) and writes C that
 * way with OUT_SPLIT (lo plane dim[4] elements after C); LAYERNORM with OUT_F32 | OUT_SPLIT writes
 * the pair to out[1] (lo plane rows*H elements after hi); ATTN_ENC with OUT_SPLIT writes the pair
 * to out[0] (lo plane batch*seq*heads*d elements after hi).
 * bf16 tensors are row-major with 16-byte aligned rows; K, lda, ldb multiples of 8.
 * LAYERNORM with OUT_F32 may also write a bf16 copy to out[1] (NULL = none).
 */
typedef struct lithos_op {
    int32_t  kind;
    uint32_t flags;
    int32_t  op_id;         /* caller's label, echoed in traces; not interpreted */
    int32_t  tile;
    int64_t  dim[8];
    int64_t  ld[4];
    float    fparam[4];
    const void* in[6];      /* device */
    void*    out[2];        /* device */
} lithos_op_t;

/* ---- context ----------------------------------------------------------- */

typedef struct lithos_config {
    double   atom_duration_us;   /* Section 4.4 'Operation': target atom length; default 250 */
    int32_t  max_outstanding;    /* Section 4.3: atoms a tenant may have in flight; default 2 */
    int32_t  max_outstanding_hp; /* same limit for LITHOS_CLASS_HP tenants; 0 = use max_outstanding */
    int32_t  steal;              /* Section 4.3 'TPC Stealing' on/off; default 1 */
    int32_t  atomize;            /* Section 4.4 on/off; default 1 */
    int32_t  xcd_remap;          /* logical-block remap that undoes round-robin XCD placement; default 1 */
    int32_t  prelude;            /* Algorithm 1 as printed: every atom launches the WHOLE grid and the blocks
                                    outside [lo,hi) exit at once (what a kernel the library does not own
                                    would need); default 0 = an atom launches exactly hi-lo workgroups that
                                    remap themselves.  Same results bit for bit; kept to measure the
                                    early-exit traffic of Section 4.4 'Performance Optimizations' */
    double   ema_alpha;          /* Section 4.7 predictor smoothing; default 0.25 */
    double   rightsize_slip;     /* Section 4.5 'Operation' in the dispatcher: latency slip k >= 1 (the paper
                                    evaluates 1.1); 0 = off (default).  When a kernel could run on its quota
                                    plus borrowed CUs, the occupancy filter (blocks / resident blocks per CU)
                                    and the model l = m/t + b, fitted to the predictor's latencies of that
                                    kernel on the two CU sets, decide whether the wider set is taken: it is
                                    not if the kernel cannot fill more than the quota, or if the model puts
                                    the quota within k of the wider set's latency.  Decided once per kernel;
                                    its atoms inherit the choice.  The model needs the kernel's latency on
                                    both sets: it borrows until the wider set has been measured, then runs
                                    on the quota once. */
} lithos_config_t;

typedef struct lithos_devinfo {
    int32_t n_cu;            /* compute units */
    int32_t n_xcd;           /* accelerator dies */
    int32_t cu_per_xcd;
    int32_t wave_size;
    int32_t lds_bytes_per_cu;
    int32_t clock_khz;
    int32_t mask_bits_interleaved; /* CU-mask bit i addresses die i % n_xcd (1) or die i / cu_per_xcd (0); probed at init */
    char    arch[32];
} lithos_devinfo_t;

/* cfg may be NULL (defaults).  device is a HIP ordinal. */
int lithos_init(int device, const lithos_config_t* cfg, lithos_ctx_t** out);
int lithos_shutdown(lithos_ctx_t* ctx);
int lithos_device_info(lithos_ctx_t* ctx, lithos_devinfo_t* out);
const char* lithos_last_error(void);

/* ---- CU partitions (the unit of Section 4.2 'Compute Quotas') ----------- */

#define LITHOS_MASK_STRIPED   0   /* n_cus spread evenly over all XCDs */
#define LITHOS_MASK_WHOLE_XCD 1   /* n_cus taken XCD by XCD (n_cus multiple of cu_per_xcd) */

/* Fill mask_out[LITHOS_MASK_WORDS] with n_cus CUs, skipping the first
 * `first` CUs of the same policy's enumeration (so two calls with
 * first=0,n=64 and first=64,n=192 give disjoint masks). */
int lithos_make_mask(lithos_ctx_t* ctx, int n_cus, int policy, int first, uint32_t* mask_out);

/* A partition owns one CU-masked HIP queue.  mask_words <= LITHOS_MASK_WORDS. */
int lithos_create_partition(lithos_ctx_t* ctx, const uint32_t* cu_mask, uint32_t mask_words,
                            lithos_partition_t** out);
int lithos_destroy_partition(lithos_partition_t* p);
int lithos_partition_cus(const lithos_partition_t* p, int* n_cus_out);
/* the partition's HIP stream, as a hipStream_t (for event timing by the caller).
 * lithos_tenant_create may replace it (see lithos_partitions_coupled): ask again
 * after tenants have been created. */
int lithos_partition_stream(const lithos_partition_t* p, void** stream_out);

/* Do the two partitions' queues share a command-processor pipe?  Measured: a grid
 * with more workgroups than `busy`'s CUs hold at once is started on `busy`, then a
 * one-block kernel on `probe`; *coupled_out = 1 if the latter had to wait for the
 * grid to be dispatched.  Both queues must be idle.  Coupled queues are legal but
 * delay each other by whole kernels; lithos_tenant_create replaces a quota
 * partition's queue (same mask) until it is independent of the other tenants'.
 * A queue's pipe follows from its position among the process's live queues, so
 * queues retired while tenants exist are kept until the last tenant is destroyed;
 * queues that other code in the process destroys can still move ours. */
int lithos_partitions_coupled(lithos_ctx_t* ctx, const lithos_partition_t* busy, const lithos_partition_t* probe,
                              int* coupled_out);

/* Run `n_wg` probe workgroups on the partition; xcd_out/cu_out[n_wg] receive
 * the die and the (shader-engine, array, CU) hardware id each one ran on. */
int lithos_probe_partition(lithos_ctx_t* ctx, const lithos_partition_t* p, uint32_t n_wg,
                           uint32_t* xcd_out, uint32_t* hwid_out);

/* ---- atomized launch (Section 4.4, Algorithm 1) -------------------------- */

/* Logical grid of an operator and how many of its workgroups fit on one CU. */
int lithos_op_grid(lithos_ctx_t* ctx, const lithos_op_t* op, lithos_dim3* grid_out,
                   uint32_t* wg_per_cu_out);

/* For a GEMM whose output has too few tiles to fill `n_cus` compute units (a weight gradient:
 * small M x N, long K): the tile selector and the number of K slices (lithos_op_t dim[5]) that
 * put about one workgroup on every CU.  slices_out = 1: leave the GEMM whole.  Only M, N, K and
 * the flags of `op` are read; nothing is launched.  The caller then provides the fp32 planes
 * (slices * M * ldc floats) and follows the GEMM with SUM_SLICES. */
int lithos_gemm_split_hint(const lithos_op_t* op, int32_t n_cus, int32_t* tile_out, int32_t* slices_out);

/* Run `op` as ceil(total/atom_blocks) launches, atom i covering logical
 * blocks [i*atom_blocks, min((i+1)*atom_blocks, total)) of the grid numbered
 * idx = z*gy*gx + y*gx + x.  atom_blocks == 0 or >= total: one launch.
 * grid {0,0,0} = use lithos_op_grid's; otherwise it must have the same total
 * (else LITHOS_EINVAL).  Atoms are ranges of the linear index, which every
 * factorisation of that total numbers alike, so a caller's grid only has to
 * agree in its total: the operator keeps its own tile geometry.
 * part NULL = an unmasked queue.  stream (hipStream_t, may be NULL = none):
 * the first atom waits for work already queued on it and it waits for the
 * last atom, so the caller's own stream work orders with the launch, and
 * launches on different partitions that name the same stream run in call
 * order.  NULL is "no ordering stream", not the legacy default stream: work
 * on the default stream (torch's default) has to be drained by the caller,
 * or moved to a created stream whose handle is passed here.  Every such hop
 * between queues costs an event round trip (tens of microseconds).
 * Returns after enqueueing; errors in shape/alignment are reported before
 * anything is launched.  If a launch fails after some atoms were enqueued,
 * the ordering stream is still made to wait for those.  Thread-safe: calls
 * on one context are serialised inside the library. */
int lithos_launch_atomized(lithos_ctx_t* ctx, const lithos_op_t* op, lithos_dim3 grid,
                           uint32_t atom_blocks, const lithos_partition_t* part, void* stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): split decode attention with the library's own workspace.
 * `op` is an ATTN_DEC descriptor with splits >= 2 and in[3] == NULL.  The key ranges' partial
 * softmaxes go to a fixed device array inside the library instead of a caller's workspace, and the
 * merge step follows on the same queue: the call does what lithos_launch_atomized(ATTN_DEC with a
 * workspace) followed by lithos_launch_atomized(ATTN_MERGE) does, with the same kernels and bit for
 * bit the same out[0].  atom_blocks cuts the ATTN_DEC launch as in lithos_launch_atomized (the
 * merge runs whole); part and stream have the same meaning as there.
 * Limit: batch * n_q * splits * (d + 2) <= LITHOS_STATIC_SCRATCH_FLOATS, else LITHOS_ELIMIT and
 * nothing is launched.  The array (8 MiB per GPU the library was initialised on, held until the
 * process ends) is shared by every call on that GPU and keeps the last call's contents; nothing in
 * it has to start at zero, since every slot that the merge reads is written first.  Calls that
 * overlap on one GPU (from two threads, or on two partitions without a common ordering stream)
 * race on it: the caller serialises them.  The call itself allocates and frees nothing. */
#define LITHOS_STATIC_SCRATCH_FLOATS (2u << 20)
int lithos_launch_attn_dec_static(lithos_ctx_t* ctx, const lithos_op_t* op, uint32_t atom_blocks,
                                  const lithos_partition_t* part, void* stream);

/* Same, for an explicit block range [lo,hi) only (one atom). */
int lithos_launch_atom(lithos_ctx_t* ctx, const lithos_op_t* op, uint32_t lo, uint32_t hi,
                       const lithos_partition_t* part);

/* Wait until everything enqueued on the partition (NULL: the unmasked queue) is done. */
int lithos_partition_sync(lithos_ctx_t* ctx, const lithos_partition_t* part);

/* Exactly-once instrumentation: while set (non-NULL), every workgroup adds 1
 * to dev_counters[logical block index] (device pointer, n uint32). */
int lithos_debug_block_counters(lithos_ctx_t* ctx, uint32_t* dev_counters, uint32_t n);

/* ---- right-sizing (Section 4.5; sweep of Section 7.2's kind) ------------- */

typedef struct lithos_rightsize_result {
    int32_t n_points;
    int32_t cus[LITHOS_MAX_SWEEP];
    double  median_us[LITHOS_MAX_SWEEP];
    int32_t chosen_cus;          /* smallest CU count within (1+slowdown) of the largest count's latency */
    double  chosen_us;
    double  full_us;
    int32_t occupancy_bound_cus; /* ceil(total blocks / resident blocks per CU), Section 4.5 'Filtering Outliers' */
    double  model_m, model_b;    /* l = m/t + b through the smallest and largest sweep points */
    int32_t model_cus;           /* smallest t with l(t) <= (1+slowdown) l(T) under that model */
    int32_t online_cus;          /* Section 4.5 'Operation' with k = 1+slowdown: the occupancy bound if it is below
                                    the largest count, else model_cus */
} lithos_rightsize_result_t;

/* Time `op` (unatomized) on striped masks of cu_lo, cu_lo+cu_step, ... cu_hi
 * CUs, `warmup` untimed then `reps` timed launches each (device timestamps). */
int lithos_rightsize(lithos_ctx_t* ctx, const lithos_op_t* op, int cu_lo, int cu_hi, int cu_step,
                     int warmup, int reps, double slowdown, lithos_rightsize_result_t* out);

/* Time `reps` launches of `op` cut in atoms of atom_blocks (0 = whole) on the
 * partition's queue (NULL: the unmasked queue), each launch bracketed by
 * device time stamps on that queue; `warmup` untimed launches first.
 * Mean and median of the per-launch durations in microseconds.  This is the
 * measurement behind the atom-overhead figure: (atomized - whole) / whole. */
int lithos_time_launch(lithos_ctx_t* ctx, const lithos_op_t* op, uint32_t atom_blocks,
                       const lithos_partition_t* part, int warmup, int reps,
                       double* mean_us_out, double* median_us_out);

/* ---- tenants and the spatial scheduler (Sections 4.2, 4.3, 4.7) ---------- */

#define LITHOS_CLASS_HP 0
#define LITHOS_CLASS_BE 1

typedef struct lithos_stats {
    uint64_t kernels;        /* kernels dispatched */
    uint64_t atoms;          /* atoms launched */
    uint64_t stolen_atoms;   /* "steals": atoms launched on a mask wider than the tenant's quota (Section 4.3
                                'TPC Stealing') */
    uint64_t revocations;    /* atom boundaries at which a kernel's next atom lost CUs that its previous atom
                                had borrowed, because their owner has work again or their timers are not free
                                (Section 4.4 'Operation', second paragraph: stealing stops for the thief's
                                later atoms; atoms in flight run to completion) */
    uint64_t rightsized_kernels; /* kernels that Section 4.5's rule kept on their quota although CUs could be borrowed */
    uint64_t predictions;    /* atoms launched with a prediction */
    uint64_t mispredicts;    /* |predicted - measured| > 50 us (Section 7.4) */
    double   abs_err_sum_us;
} lithos_stats_t;

/* quota: the partition whose CUs the tenant is guaranteed.  Quotas of
 * different tenants must be disjoint.  Call while the context's queues are idle:
 * the partition's queue may be re-created (same CU mask) so that it does not share
 * a command-processor pipe with another tenant's queue, and the queues for
 * quota + stolen CUs of each pair of tenants are created here.  quota NULL makes a pass-through tenant:
 * every kernel is launched whole, at submission, on an unmasked queue of the
 * tenant's own (the unpartitioned co-execution that the scheduler is compared
 * with). */
int lithos_tenant_create(lithos_ctx_t* ctx, int cls, const lithos_partition_t* quota,
                         lithos_tenant_t** out);
int lithos_tenant_destroy(lithos_tenant_t* t);
/* Enqueue on the tenant's launch queue and return at once (Section 4.2).
 * The op descriptor is copied.  ticket_out (may be NULL) identifies the kernel. */
int lithos_submit(lithos_tenant_t* t, const lithos_op_t* op, uint64_t* ticket_out);
/* Batch boundary: later kernels restart at ordinal 0 (Section 4.7).  Does not block. */
int lithos_sync_mark(lithos_tenant_t* t);
/* Block until every kernel submitted so far has completed; implies lithos_sync_mark. */
int lithos_sync(lithos_tenant_t* t);
int lithos_poll(lithos_tenant_t* t, uint64_t ticket, int* done_out);
int lithos_tenant_stats(lithos_tenant_t* t, lithos_stats_t* out);
/* Totals over every tenant the context has had (destroyed ones included): kernels, atoms launched,
 * steals, revocations, predictions and mispredictions. */
int lithos_stats(lithos_ctx_t* ctx, lithos_stats_t* out);

/* ---- load generators (native, so that two tenants do not share an interpreter lock) */
/* These stand in for the paper's clients (Section 7.1: high-priority
 * applications follow a Poisson load, best-effort ones run in a closed loop). */

typedef struct lithos_driver lithos_driver_t;

/* Open loop, in the calling thread: request r is submitted at arrivals_s[r]
 * seconds after the call starts (never earlier; later only if the thread is
 * late), as the ops_per_request operators ops[(r % n_variants)*ops_per_request ...]
 * followed by a batch boundary.  latency_us_out[r] = completion - scheduled
 * arrival.  Returns when every request has completed. */
int lithos_drive_open_loop(lithos_tenant_t* t, const lithos_op_t* ops, int ops_per_request, int n_variants,
                           const double* arrivals_s, int n_requests, double* latency_us_out);

/* Closed loop on a thread of its own: keeps `depth` iterations (each the
 * ops_per_iter operators followed by a batch boundary) in flight until stopped. */
int lithos_drive_closed_loop_start(lithos_tenant_t* t, const lithos_op_t* ops, int ops_per_iter, int depth,
                                   lithos_driver_t** out);
/* Stops after the iterations in flight; reports completed iterations and the
 * wall time between the first submission and the last completion. */
int lithos_drive_closed_loop_stop(lithos_driver_t* d, uint64_t* iterations_out, double* seconds_out);

/* ---- scheduler policy core, steppable with a caller-supplied clock -------- */
/* The same decision code the dispatcher threads run, without a device: the
 * caller plays device and clock.  Used to check the policy on a CPU. */

typedef struct lithos_core lithos_core_t;

typedef struct lithos_core_atom {
    uint64_t atom_id;
    int32_t  tenant;
    uint64_t kernel_id;
    int32_t  ordinal;
    uint32_t lo, hi;
    uint32_t group_mask;     /* bit g = CU group g (cus_per_group CUs each) */
    int32_t  stolen;
    int32_t  has_prediction;
    double   predicted_us;
} lithos_core_atom_t;

int lithos_core_create(const lithos_config_t* cfg, int n_groups, int cus_per_group, lithos_core_t** out);
int lithos_core_destroy(lithos_core_t* c);
int lithos_core_add_tenant(lithos_core_t* c, int cls, uint32_t quota_groups, int* tenant_out);
int lithos_core_submit(lithos_core_t* c, int tenant, uint32_t total_blocks, uint32_t wg_per_cu,
                       uint64_t* kernel_id_out);
int lithos_core_sync_mark(lithos_core_t* c, int tenant);
/* Next atom the tenant should launch at time now_us; *have_out = 0 if none
 * (nothing queued, or the outstanding limit is reached). */
int lithos_core_next_atom(lithos_core_t* c, int tenant, double now_us, lithos_core_atom_t* atom_out,
                          int* have_out);
int lithos_core_complete(lithos_core_t* c, uint64_t atom_id, double now_us, double measured_us);
int lithos_core_stats(lithos_core_t* c, int tenant, lithos_stats_t* out);

#ifdef __cplusplus
}
#endif
#endif /* LITHOS_H */
