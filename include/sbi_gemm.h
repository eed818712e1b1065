/*
 * sbi_gemm.h - C ABI of the MI355X (gfx950) small-batch inference GeMM library.
 *
 * The operation is the one the DeepSpeed Inference paper (arXiv 2207.00032) builds its
 * latency work on: at small batch a transformer layer's linear layers are bound by the
 * time it takes to read the weights once (Sec. I, "Latency Challenges"), so the GeMM
 *
 *     Y[B,N] = epilogue( X[B,K] . W[K,N] + bias[N] )          B = 1 .. 64
 *
 * is a weight-streaming kernel (Sec. III-C, "SBI-GeMM").  W is fp16, products are
 * accumulated in fp32, Y is fp16 (one round-to-nearest-even step at the very end).
 * The epilogue is the element-wise tail the paper fuses into the producing kernel
 * (Sec. III-B fusion rule; Sec. III-D region 4, "bias and residual addition").
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers into memory owned by the caller; the
 *     library never allocates, frees or retains device memory.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).  All
 *     work is enqueued on it and no call synchronises, except sbi_gemm_layout_check.
 *   - Arguments are validated on the host before any GPU call; a failed validation
 *     enqueues nothing.  No exception crosses the boundary; the result is an sbi_status.
 *   - Mutable state: each thread keeps a small memo of the launch plans it computed last; the
 *     plans measured by sbi_layer_tune / sbi_gemm_tune live in a process-wide table behind a mutex.
 *     Calls on different streams may overlap as long as they do not share a workspace.
 */
#ifndef SBI_GEMM_H
#define SBI_GEMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SBI_MAX_BATCH 64

typedef enum sbi_status {
    SBI_OK = 0,
    SBI_ERR_NULL = 1,            /* a required pointer is NULL */
    SBI_ERR_SHAPE = 2,           /* K or N < 1, or too large for 32-bit tile counts */
    SBI_ERR_ALIGN = 3,           /* a pointer is not aligned as documented */
    SBI_ERR_BATCH = 4,           /* B outside 1..SBI_MAX_BATCH */
    SBI_ERR_LAYOUT_MISMATCH = 5, /* laid-out buffer header does not match (K, N) */
    SBI_ERR_WORKSPACE = 6,       /* workspace missing or too small */
    SBI_ERR_EPILOGUE = 7,        /* unknown epilogue, or its bias/residual pointer is NULL */
    SBI_ERR_HIP = 8,             /* the HIP runtime reported an error */
    SBI_ERR_OVERLAP = 9,         /* Y overlaps X */
    SBI_ERR_TUNING = 10          /* an explicit tuning request is not supported */
} sbi_status;

/* v = acc (+ bias[n]);  GELU: v = 0.5 v (1 + erf(v / sqrt 2));  RESIDUAL: v += R[b,n]. */
typedef enum sbi_epilogue {
    SBI_EPI_NONE = 0,
    SBI_EPI_BIAS = 1,
    SBI_EPI_BIAS_GELU = 2,
    SBI_EPI_BIAS_RESIDUAL = 3,
    SBI_EPI_GELU = 4,
    SBI_EPI_RESIDUAL = 5
} sbi_epilogue;

/* Which kernel family executes the contraction. */
typedef enum sbi_path {
    SBI_PATH_AUTO = 0,   /* the batch-size dispatcher decides */
    SBI_PATH_STREAM = 1, /* vector-ALU dot-product kernel, one block per (panel, k-range), B <= 8 */
    SBI_PATH_MFMA = 2,   /* matrix-core (MFMA fp16 16x16x32) kernel, one block per (panel, k-range) */
    SBI_PATH_STREAMK = 3 /* matrix-core kernel with the weight stream cut into equal ranges, one per
                            wavefront; needs K % 8 == 0; the only path that groups a layer's GeMMs */
} sbi_path;

/* Optional overrides for sbi_gemm_ex / sbi_gemm_plan; a zero field means "automatic". */
typedef struct sbi_tuning {
    int32_t path;    /* sbi_path */
    int32_t split_k; /* blocks that share one 64-column panel's K range (STREAM / MFMA paths) */
    int32_t waves;   /* wavefronts per block: 4 or 8 */
    int32_t depth;   /* k-steps of W each wavefront keeps in flight: 2 (MFMA path), 4 or 8 */
    int32_t blocks;  /* STREAMK path: upper bound on the number of thread blocks */
    int32_t panels;  /* MFMA path: 64-column panels per block, 1 or 2 (2: X is staged once for 128
                        columns; for larger batches.  With waves = 8: depth 2 - every wave streams both
                        panels; depth 4, B > 16 - two groups of four waves, one panel each) */
    int32_t layernorm; /* sbi_gemm_plan: nonzero plans the launch sbi_gemm_ln makes (layer-norm fused
                          in front: MFMA path, one panel per block, K % 8 == 0, (waves, depth) one of
                          (4,2), (4,4), (8,4)); sbi_gemm_ex rejects it, sbi_gemm_ln implies it */
    int32_t int8;      /* sbi_gemm_plan: nonzero plans the launch sbi_gemm_i8 makes (MFMA path, K % 16 == 0;
                          (waves, depth) one of (4,2), (4,4), (8,4) with one panel per block, or (8,2) with two
                          panels per block for B > 8); sbi_gemm_i8 implies it.  Together with layernorm: the
                          launches sbi_gemm_i8_ln makes */
} sbi_tuning;

/* What the dispatcher decided for a problem (for reports and tests). */
typedef struct sbi_plan {
    int32_t path;        /* SBI_PATH_STREAM, SBI_PATH_MFMA or SBI_PATH_STREAMK */
    int32_t waves;       /* wavefronts per block */
    int32_t depth;       /* W k-steps in flight per wavefront */
    int32_t split_k;     /* blocks per panel (1 = no cross-block reduction); 0 on the STREAMK path */
    int32_t ksteps_per_split; /* k-steps handled by one block (STREAMK: 4 KiB units per wavefront) */
    int32_t ksteps_per_chunk; /* k-steps of X staged in LDS at a time; 0 on the STREAMK path */
    int32_t grid;        /* thread blocks launched */
    int32_t block;       /* threads per block */
    int32_t panels;      /* 64-column panels per block (MFMA path), else 1 */
    int32_t reserved;
    int64_t lds_bytes;   /* dynamic LDS per block */
    int64_t workspace_bytes; /* workspace this plan needs (0 when split_k == 1) */
} sbi_plan;

/*
 * Size in bytes of the laid-out copy of a [K,N] fp16 matrix: a 256-byte header followed
 * by ceil(N/64) * KS k-steps of 4 KiB (zero padded), KS = ceil(K/32) rounded up to a
 * multiple of 8.  Returns 0 for a bad shape.
 */
size_t sbi_gemm_layout_bytes(int64_t K, int64_t N);

/*
 * Upper bound of the workspace sbi_gemm (automatic dispatch) needs for (B, K, N), in bytes;
 * may be 0.  The workspace holds a fixed 256 KiB region of arrival counters (one per
 * 64-column panel) followed by the cross-block partial sums.
 * It MUST be zero-filled once by the caller before its first use; the library
 * leaves the counters zero after every call, so one workspace can serve any sequence
 * of calls on one stream.  Two calls that may run concurrently must not share it.
 */
size_t sbi_gemm_workspace_bytes(int64_t B, int64_t K, int64_t N);

/*
 * One-time weight pre-layout (paper Sec. III-C, "Leveraging Full Cache-line": re-tile W
 * at initialisation so that every thread reads several consecutive input-dimension
 * elements of its column in one access).  Here one lane of a 64-wide wavefront owns
 * 8 consecutive k of one column (one 128-bit load), a wavefront load is a contiguous
 * 1 KiB tile of 16 columns x 32 k, and the four tiles of a 64-column panel are adjacent:
 *   half index of W[k][n] after the header =
 *     ((((n/64)*KS + k/32)*4 + (n%64)/16)*64 + ((k%32)/8)*16 + n%16)*8 + k%8,
 *   KS = ceil(K/32) rounded up to a multiple of 8 (so K is zero padded to a multiple of 256).
 * W_rowmajor: device, fp16 [K,N] contiguous (ld = N), 2-byte aligned.
 * W_laid_out: device, 256-byte aligned, laid_out_bytes >= sbi_gemm_layout_bytes(K,N).
 * The source may be freed once the stream has executed the call.  Pure permutation plus
 * zero padding: sbi_gemm_unlayout_weights restores the original bits.
 */
sbi_status sbi_gemm_layout_weights(const void* W_rowmajor, int64_t K, int64_t N,
                                   void* W_laid_out, size_t laid_out_bytes, void* hip_stream);

/* Inverse of sbi_gemm_layout_weights: writes fp16 [K,N] row-major into W_rowmajor. */
sbi_status sbi_gemm_unlayout_weights(const void* W_laid_out, int64_t K, int64_t N,
                                     void* W_rowmajor, void* hip_stream);

/*
 * Reads the header of a laid-out buffer back to the host (synchronises the stream) and
 * returns SBI_OK if it was written by this library version for exactly (K, N),
 * SBI_ERR_LAYOUT_MISMATCH otherwise.  sbi_gemm itself trusts its W_laid_out argument.
 */
sbi_status sbi_gemm_layout_check(const void* W_laid_out, int64_t K, int64_t N, void* hip_stream);

/*
 * The small-batch GeMM (paper Sec. III-C; epilogue: Sec. III-D region 4).
 *   W_laid_out  device, from sbi_gemm_layout_weights for the same (K, N)
 *   X           device, fp16 [B,K] row-major contiguous; 16-byte aligned when K % 8 == 0,
 *               2-byte aligned otherwise
 *   bias        device, fp16 [N], required by the BIAS* epilogues, ignored otherwise
 *   residual    device, fp16 [B,N], required by the *RESIDUAL epilogues; may alias Y
 *   Y           device, fp16 [B,N] row-major contiguous, 4-byte aligned; must not overlap X
 *   workspace   device, 256-byte aligned, zero-filled once before first use;
 *               workspace_bytes >= sbi_gemm_workspace_bytes(B,K,N); may be NULL when that is 0
 * Results are deterministic: the same inputs give the same bits on every call.
 */
sbi_status sbi_gemm(const void* W_laid_out, int64_t K, int64_t N,
                    const void* X, int64_t B,
                    const void* bias, const void* residual, sbi_epilogue epi,
                    void* Y, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * sbi_gemm for callers that cannot provide (or allocate) a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same operation, same kernels,
 * same launch plan and therefore the same bits as sbi_gemm; the arrival counters and cross-block
 * partial sums live in a device array of SBI_STATIC_SCRATCH_BYTES that is part of the library's
 * code object (every GPU the library runs on holds its own copy until the process ends).  The
 * call allocates and frees nothing.
 *   - A problem whose plan needs more than SBI_STATIC_SCRATCH_BYTES of workspace
 *     (sbi_gemm_workspace_bytes(B,K,N); e.g. B = 64 with K = 131072, N = 12288) is refused with
 *     SBI_ERR_WORKSPACE and nothing is enqueued: use sbi_gemm with a workspace for those.
 *   - All calls on one GPU share that GPU's array: two calls that may run concurrently on one GPU
 *     (different streams, different host threads) race on it.  Calls on one stream are safe.
 *   - The first call on a GPU looks the array's address up and enqueues a small kernel on
 *     `hip_stream` that clears the counters; make that first call outside graph capture.
 * Arguments as for sbi_gemm.
 */
#define SBI_STATIC_SCRATCH_BYTES (16u << 20)
sbi_status sbi_gemm_static(const void* W_laid_out, int64_t K, int64_t N,
                           const void* X, int64_t B,
                           const void* bias, const void* residual, sbi_epilogue epi,
                           void* Y, void* hip_stream);

/* sbi_gemm with explicit tuning (NULL = automatic).  Workspace need: see sbi_gemm_plan. */
sbi_status sbi_gemm_ex(const void* W_laid_out, int64_t K, int64_t N,
                       const void* X, int64_t B,
                       const void* bias, const void* residual, sbi_epilogue epi,
                       void* Y, void* workspace, size_t workspace_bytes, void* hip_stream,
                       const sbi_tuning* tuning);

/*
 * Layer normalisation fused in front of the GeMM (paper Sec. III-D: regions 1 and 3 of the
 * fused layer start with "input layer-norm" and run into the QKV / intermediate GeMM, with
 * the input batch broadcast to every thread block so that no kernel boundary is needed):
 *
 *     mean_b = (1/K) sum_k X[b,k]          var_b = (1/K) sum_k (X[b,k] - mean_b)^2
 *     Xn[b,k] = fp16( (X[b,k] - mean_b) / sqrt(var_b + eps) * gamma[k] + beta[k] )
 *     Y = epilogue( Xn . W + bias )
 *
 * Up to 8 rows (4 on launches of a gigabyte and more) every thread block recomputes the B row
 * statistics (fp32, two passes) and normalises its share of X on the way into the matrix-core
 * operand; above that a kernel of its own normalises the rows once into the workspace and the
 * plain GeMM kernels run on the result (with automatic tuning; an explicit `tuning` keeps the
 * fused form).  `moments` shorten the statistics of the fused form only; the separate kernel
 * recomputes them from the rows.  Either way Xn is rounded to fp16 once: it is the matrix-core
 * operand.
 *   gamma, beta  device, fp16 [K], 16-byte aligned
 *   eps          finite, >= 0
 * Needs K % 8 == 0 (SBI_ERR_SHAPE otherwise).  Everything else as for sbi_gemm_ex; `tuning`
 * may be NULL.  Workspace need: sbi_gemm_ln_workspace_bytes, or sbi_gemm_plan with
 * tuning->layernorm set (it can differ from the plain GeMM's).
 */
typedef struct sbi_layernorm {
    const void* gamma;
    const void* beta;
    float eps;
    const void* moments; /* optional (NULL: the statistics are computed from X): per-panel row moments of X
                            as written by sbi_gemm_moments for the GeMM that produced X; needs K % 64 == 0 */
} sbi_layernorm;

sbi_status sbi_gemm_ln(const void* W_laid_out, int64_t K, int64_t N,
                       const void* X, int64_t B, const sbi_layernorm* ln,
                       const void* bias, const void* residual, sbi_epilogue epi,
                       void* Y, void* workspace, size_t workspace_bytes, void* hip_stream,
                       const sbi_tuning* tuning);

size_t sbi_gemm_ln_workspace_bytes(int64_t B, int64_t K, int64_t N);

/*
 * The residual path of the fused layer (paper Sec. III-B fusion rule, Sec. III-D: "bias and
 * residual addition" run into the next region, which starts with a layer-norm): a GeMM whose
 * epilogue, besides Y = epilogue(X.W + bias (+ residual)), leaves what the FOLLOWING layer-norm
 * needs of Y.  A full normalisation needs whole rows, which are spread over the 64-column panels
 * of different thread blocks, so the epilogue finishes each panel's part:
 *
 *     row_moments[b][p] = ( mean, sum of squared deviations from that mean )
 *                         of the stored fp16 values Y[b, 64p .. min(64p+64, N))      (float2)
 *
 * The consuming call (sbi_gemm_ln on Y with ln->moments = row_moments) merges a row's panels
 * exactly (mean = sum n_p mean_p / K, M2 = sum (M2_p + n_p (mean_p - mean)^2)) instead of reading
 * the row again for its statistics.  As sbi_gemm_ln (ln may be NULL: no layer-norm in front of
 * THIS GeMM), fp16 matrix-core path only.
 *   row_moments  device, 8-byte aligned, float2 [B][ceil(N/64)], written completely
 */
sbi_status sbi_gemm_moments(const void* W_laid_out, int64_t K, int64_t N,
                            const void* X, int64_t B, const sbi_layernorm* ln,
                            const void* bias, const void* residual, sbi_epilogue epi,
                            void* Y, void* row_moments, void* workspace, size_t workspace_bytes, void* hip_stream,
                            const sbi_tuning* tuning);

/*
 * INT8 GeMM (paper Sec. III-D, "Support for Different Data Types": an INT8 GeMM with the quantize
 * operation fused in front of it and the de-quantisation fused into its epilogue; Sec. III-C
 * "Leveraging Full Cache-line": INT8 gets its own, wider pre-layout).  The paper gives no
 * quantisation formula; this library uses the plain symmetric one, per output channel for the
 * weights and per row (token) for the activations, every step in IEEE binary32:
 *
 *     amax = max |v|      inv = 127 / amax      scale = amax / 127     (amax = 0: inv = scale = 0)
 *     code = clamp(rint(v * inv), -127, 127)                            (ties to even)
 *     Y[b,n] = epilogue( (sum_k Xq[b,k] * Wq[k,n]) * sx[b] * sw[n] + bias[n] )
 *
 * The integer sum is exact (int32; |sum| <= 127^2 K); the activations are quantised by the call
 * itself (up to B = 8 every block of the GeMM kernel finds the rows' maxima and quantises what it
 * stages; above that a kernel of its own writes codes and row scales to the workspace first), so
 * X, bias, residual and Y are fp16 as in sbi_gemm.  Half the weight bytes of the fp16 path are
 * streamed.
 *
 * sbi_gemm_i8_quantize_weights: W fp16 [K,N] row-major (device) -> codes Wq int8 [K,N] row-major
 *   and scales sw binary32 [N] (both device, caller-owned).  Optional: codes and scales that were
 *   produced elsewhere under the same convention can be used directly.
 * sbi_gemm_i8_layout_weights: codes [K,N] row-major -> laid-out buffer of
 *   sbi_gemm_i8_layout_bytes(K,N) bytes (256-byte aligned): 256-byte header, then per panel of 64
 *   columns and per step of 64 k four 1 KiB tiles in which lane (g, i) holds the 16 codes
 *   k = 16g..16g+15 of column i; zero padded.
 * sbi_gemm_i8: as sbi_gemm_ex with the laid-out codes and w_scales (device, binary32 [N], 4-byte
 *   aligned).  Needs K % 16 == 0 (SBI_ERR_SHAPE).  Workspace: sbi_gemm_i8_workspace_bytes.
 * sbi_gemm_i8_ln: the layer normalisation of sbi_gemm_ln in front of the INT8 GeMM (the paper's
 *   fused regions 1 and 3 start with the input layer-norm whatever the GeMM's data type):
 *       Xn = fp16( layernorm(X) )     then     Y = sbi_gemm_i8 on Xn.
 *   The fp16 value Xn[b,k] decides an integer code, so it must be THE correctly rounded value of
 *   the definition: one kernel (a block per row) evaluates the row statistics and
 *   (x - mean) / sqrt(var + eps) * gamma + beta in binary64, rounds once to fp16, quantises the row
 *   as above and leaves codes and row scales in the workspace; the INT8 GeMM kernels then run from
 *   those codes at every batch size.  ln->moments must be NULL.  Workspace: sbi_gemm_plan with
 *   tuning->int8 and tuning->layernorm both set.
 */
size_t sbi_gemm_i8_layout_bytes(int64_t K, int64_t N);
size_t sbi_gemm_i8_workspace_bytes(int64_t B, int64_t K, int64_t N);
sbi_status sbi_gemm_i8_quantize_weights(const void* W_rowmajor, int64_t K, int64_t N,
                                        void* Wq_rowmajor, void* w_scales, void* hip_stream);
sbi_status sbi_gemm_i8_layout_weights(const void* Wq_rowmajor, int64_t K, int64_t N,
                                      void* W_laid_out, size_t laid_out_bytes, void* hip_stream);
sbi_status sbi_gemm_i8_layout_check(const void* W_laid_out, int64_t K, int64_t N, void* hip_stream);
sbi_status sbi_gemm_i8(const void* W_laid_out, const void* w_scales, int64_t K, int64_t N,
                       const void* X, int64_t B,
                       const void* bias, const void* residual, sbi_epilogue epi,
                       void* Y, void* workspace, size_t workspace_bytes, void* hip_stream,
                       const sbi_tuning* tuning);
sbi_status sbi_gemm_i8_ln(const void* W_laid_out, const void* w_scales, int64_t K, int64_t N,
                          const void* X, int64_t B, const sbi_layernorm* ln,
                          const void* bias, const void* residual, sbi_epilogue epi,
                          void* Y, void* workspace, size_t workspace_bytes, void* hip_stream,
                          const sbi_tuning* tuning);

/* Host-only: the launch the dispatcher would make for (B, K, N) under `tuning` (or NULL). */
sbi_status sbi_gemm_plan(int64_t B, int64_t K, int64_t N, const sbi_tuning* tuning, sbi_plan* plan);

/*
 * One transformer layer's four linear layers (paper Sec. III-D, Fig. 1(c): QKV,
 * attention output, FFN1 "intermediate" GeMM, FFN2 with bias and residual addition).
 * Shapes: QKV [h, n_qkv]; out [k_out, h]; FFN1 [h, n_ffn1]; FFN2 [k_ffn2, h] - this
 * covers a full layer (n_qkv = 3h, k_out = h, n_ffn1 = k_ffn2 = 4h) and a tensor-parallel
 * slice of one.  W* are laid-out buffers; a NULL bias pointer drops that bias.
 */
typedef struct sbi_layer {
    const void *Wqkv, *Wout, *Wffn1, *Wffn2; /* device, laid out */
    const void *bqkv, *bout, *bffn1, *bffn2; /* device fp16 or NULL */
    int64_t h, n_qkv, k_out, n_ffn1, k_ffn2;
    int32_t ffn1_gelu;                        /* nonzero: GeLU after FFN1's bias */
    /* optional layer-norms fused in front of QKV (ln1, over Xqkv's rows) and FFN1 (ln2, over
       Xffn1's rows), as in sbi_gemm_ln: device fp16 [h], 16-byte aligned, gamma and beta both
       set or both NULL; they need h % 8 == 0 */
    const void *ln1_gamma, *ln1_beta, *ln2_gamma, *ln2_beta;
    float ln_eps;
    /* INT8 layer: all four set (device, binary32 per-column scales [n_qkv], [h], [n_ffn1], [h]) means
       W* are laid-out int8 codes (sbi_gemm_i8_layout_weights) and the GeMMs run as sbi_gemm_i8;
       all four NULL: fp16.  Needs h, k_out, k_ffn2 % 16 == 0.  With ln1/ln2: as sbi_gemm_i8_ln. */
    const void *sqkv, *sout, *sffn1, *sffn2;
} sbi_layer;

/*
 * Enqueues the four GeMMs on one stream:
 *   Yqkv  [B,n_qkv] = LN1?(Xqkv[B,h]) . Wqkv (+ bqkv)
 *   Yout  [B,h]     = Xout[B,k_out] . Wout (+ bout)
 *   Yffn1 [B,n_ffn1]= act(LN2?(Xffn1[B,h]) . Wffn1 (+ bffn1))
 *   Yffn2 [B,h]     = Xffn2[B,k_ffn2] . Wffn2 (+ bffn2) (+ residual[B,h])
 * Xffn2 == NULL chains FFN1's output (requires n_ffn1 == k_ffn2).  residual may be NULL.
 * workspace_bytes >= sbi_layer_workspace_bytes(L, B) always suffices (a call checks against what
 * its own launches need, which is never more).
 */
sbi_status sbi_layer_gemms(const sbi_layer* L, int64_t B,
                           const void* Xqkv, const void* Xout, const void* Xffn1, const void* Xffn2,
                           const void* residual,
                           void* Yqkv, void* Yout, void* Yffn1, void* Yffn2,
                           void* workspace, size_t workspace_bytes, void* hip_stream);

size_t sbi_layer_workspace_bytes(const sbi_layer* L, int64_t B);

/*
 * Host-only: the launch sbi_layer_gemms makes for the layer's independent GeMMs (`chained`
 * nonzero: QKV, attention output, FFN1; zero: all four).  plans[g] receives GeMM g's share:
 * its split, k-steps per block, X chunk and number of blocks; waves, depth, block and
 * lds_bytes are those of the common launch.  *total_grid receives the launch's block count.
 */
sbi_status sbi_layer_plan(const sbi_layer* L, int64_t B, int32_t chained, sbi_plan plans[4], int32_t* total_grid);

/*
 * Measured launch plans.  The dispatcher ranks block shapes and splits with a cost model; which of
 * its near-best candidates is fastest depends on the shapes of the launch and on the machine, so
 * a caller that runs the same launches many times (every layer of a model, every generated token)
 * can have them measured once, at model load: the call runs the launch under each candidate plan
 * the model puts within 30 % of its best estimate (at most 48 distinct plans, about 30 launches
 * each), on the caller's own tensors, and records the fastest for (B, shapes, data type, layer-norm
 * or not) in a process-wide table that every later plan, workspace-size and launch call of this
 * library consults first (a candidate displaces the model's own pick only if it is more than 1 %
 * faster: less than that is the spread of such measurements).  This serves the paper's aim for the
 * small-batch GeMM - a launch that takes no longer than reading the weights once (Sec. I, latency
 * challenges; Sec. III-C picks its tiling by problem size): here the tiling is chosen by measurement.
 *   layers / W_laid_out  n weight sets of ONE shape (a model's consecutive layers): trial launch i uses
 *                        set i mod n, so that with enough sets the weights come from HBM as they do in
 *                        the model, not from the last-level cache
 *   workspace            as for the call being tuned; candidates that would need more are left out
 *   report               optional: how many plans were tried, the winner, its time and the time of the
 *                        model's own pick
 * The call synchronises the stream (it times with events) and creates and destroys two events; it
 * allocates no device memory.  The outputs hold valid results of the last trial.  Results are
 * deterministic per plan; a different plan may round differently in the last bit (another order of
 * the fp32 additions).  Not for use under graph capture.
 * sbi_gemm_tune tunes the plain fp16 sbi_gemm; sbi_layer_tune the launch sbi_layer_gemms makes for
 * the layer's independent GeMMs (with Xffn2 == NULL: QKV, attention output, FFN1).
 */
typedef struct sbi_tune_report {
    int32_t candidates;     /* distinct plans measured */
    int32_t waves, depth, panels, block_ksteps; /* the winner: block shape and common block size */
    float us_best;          /* its time per launch */
    float us_model;         /* time per launch of the plan the cost model ranks first */
} sbi_tune_report;

sbi_status sbi_layer_tune(const sbi_layer* layers, int32_t n_layers, int64_t B,
                          const void* Xqkv, const void* Xout, const void* Xffn1, const void* Xffn2,
                          const void* residual,
                          void* Yqkv, void* Yout, void* Yffn1, void* Yffn2,
                          void* workspace, size_t workspace_bytes, void* hip_stream, sbi_tune_report* report);

sbi_status sbi_gemm_tune(const void* const* W_laid_out, int32_t n_weights, int64_t K, int64_t N,
                         const void* X, int64_t B,
                         const void* bias, const void* residual, sbi_epilogue epi,
                         void* Y, void* workspace, size_t workspace_bytes, void* hip_stream, sbi_tune_report* report);

/*
 * Single-token attention with a key/value cache (paper Sec. III-D region 2, "transposition plus
 * attention" in one kernel; Sec. IV: token generation re-uses the past through the KV cache and
 * computes only for the one new token).  Standard scaled dot-product attention, per sequence b
 * and head h, with the new token's query / key / value taken from the QKV GeMM's output row:
 *
 *     K[b][h][pos] = k_new,  V[b][h][pos] = v_new                      (the transposition)
 *     s_j = scale * q . K[b][h][j]        p = softmax_j(s_j)           j = 0 .. pos
 *     out[b][h*d .. h*d+d) = fp16( sum_j p_j V[b][h][j] )
 *
 *   qkv         device, fp16 [B][3][heads][head_dim] (query, key, value), 16-byte aligned
 *   k_cache,
 *   v_cache     device, fp16 [B][heads][max_seq][head_dim], 16-byte aligned, holding `pos` earlier
 *               tokens of every sequence at positions 0 .. pos-1; position `pos` is written
 *   pos         0 <= pos < max_seq: the same for all sequences of the batch
 *   scale       > 0, or 0 for 1/sqrt(head_dim)
 *   out         device, fp16 [B][heads*head_dim]
 *   workspace   device, 256-byte aligned, zero-filled once before first use,
 *               >= sbi_attn_decode_workspace_bytes(B, heads, head_dim, max_seq) (0 for short caches)
 * head_dim is 64 or 128; B <= SBI_MAX_BATCH.  Accumulation in fp32, one rounding to fp16;
 * deterministic.  Cached keys and values are read exactly once.
 */
size_t sbi_attn_decode_workspace_bytes(int64_t B, int32_t heads, int32_t head_dim, int64_t max_seq);
sbi_status sbi_attn_decode(const void* qkv, void* k_cache, void* v_cache, int64_t B, int32_t heads, int32_t head_dim,
                           int64_t max_seq, int64_t pos, float scale, void* out,
                           void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * The same attention (paper Sec. III-D region 2; Sec. IV token-generation phase) for a batch whose
 * sequences are at different lengths, as a serving batch's are: sequence b's new token goes to
 * position pos[b] of its cache and attends to positions 0 .. pos[b].
 *
 *   pos         device, int32 [B], 4-byte aligned; read by the kernel, never by the host
 *   pos_bound   host value with 0 <= pos_bound < max_seq; the caller guarantees pos[b] <= pos_bound.
 *               It sizes the launch (position ranges per sequence and head are cut for pos_bound + 1
 *               positions; a shorter sequence's surplus ranges are empty), so a tight bound is
 *               faster.  An entry outside 0 .. pos_bound is not an error the kernel can report: it is
 *               forced to the nearer end of that interval, so no entry reaches outside the caches.
 * Everything else as for sbi_attn_decode, whose result row b equals this call's when pos[b] == pos
 * (bit for bit when pos_bound == pos as well: the same ranges are summed in the same order).
 */
sbi_status sbi_attn_decode_ragged(const void* qkv, void* k_cache, void* v_cache, int64_t B, int32_t heads,
                                  int32_t head_dim, int64_t max_seq, const int32_t* pos, int64_t pos_bound, float scale,
                                  void* out, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Diagnostic (needs a GPU, enqueues nothing): vector registers per lane of the GeMM kernel variant that
 * serves `B` rows with blocks of `waves` wavefronts, a weight ring of `depth` and `panels` panels per
 * block.  flavour: 0 fp16, 1 fp16 with the layer-norm in front, 2 INT8 quantising X in the block,
 * 3 INT8 from pre-quantised codes.  *allocated is what the compiled kernel uses (the runtime's figure),
 * *assumed what the dispatcher's occupancy model takes for it: the model counts resident blocks per
 * compute unit from the latter (Sec. III-C: the kernel's schedule is chosen for the memory bandwidth it
 * reaches, which depends on how many blocks a unit holds), so the two must land in the same register
 * granule.  SBI_ERR_TUNING: no such variant.  SBI_ERR_HIP: the runtime refused the query.
 */
sbi_status sbi_kernel_registers(int64_t B, int32_t waves, int32_t depth, int32_t panels, int32_t flavour,
                                int32_t* allocated, int32_t* assumed);

const char* sbi_status_string(sbi_status s);

/* Library version: major*10000 + minor*100 + patch. */
int32_t sbi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SBI_GEMM_H */
