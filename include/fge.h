/*
 * fge.h - C ABI of the fused GEMM + activation + row-normalisation library for MI355X (gfx950).
 *
 * The operation is the fused operator chain that a kernel generator emits for a dense layer
 * followed by an activation and a row-wise reduction / normalisation (the paper's "fused
 * operations" and "normalization operations" categories, Section 3.6; the reason for fusing -
 * no intermediate memory traffic, one launch instead of several - is its Section 4.3):
 *
 *     Y   = post_scale * (alpha * X . W^T + b)          X: rows x K,  W: N x K,  b: N
 *     A   = act(Y)                                      elementwise
 *     out = rowop_N(A)                                  over the N columns of each row
 *
 * Layout.  X and W are row-major with the contraction axis K contiguous (row strides ldx,
 * ldw in elements); out is row-major rows x N (row stride ldo).  b, gamma, beta are fp32
 * vectors of length N; aux_out is an fp32 vector with one entry per row.  With batch > 1 the
 * library processes `batch` problems of M rows each that share W, b, gamma, beta; problem z
 * reads X + z*batch_stride_x, writes out + z*batch_stride_o and aux_out + z*M.
 *
 * Ownership.  Every pointer except `p` and the returned strings is DEVICE memory owned by
 * the caller.  The library allocates nothing, frees nothing and keeps no pointer after a call
 * returns; its only state is a launch counter.  `workspace` is caller-provided device scratch
 * of at least fge_workspace_bytes(); its contents need no initialisation and two launches that
 * may overlap must not share one.
 *
 * Asynchrony.  Calls only enqueue work on `stream` (a hipStream_t passed as void*; NULL is
 * the default stream) and return; they never synchronise the device.  Calls may be captured
 * into a HIP graph (nothing is allocated, no memset node is recorded); on a capturing stream
 * split rows always take the two-pass form, and fge_workspace_bytes covers both forms.
 *
 * Errors.  Every function returning int returns an fge_status.  All argument checks are done
 * on the host before anything is launched, so a non-zero status other than FGE_ERR_HIP means
 * that no work was enqueued.  FGE_ERR_UNSUPPORTED is left for requests beyond the index range
 * (more than 2^30 rows in total) and operand / output type pairs outside the set below.
 *
 * Supported set.  in_dtype in {FGE_F32, FGE_BF16, FGE_F16, FGE_F8E4M3}; out_dtype FGE_F32 or the
 * 16-bit type that goes with the operands (FGE_BF16 with fp32, bf16 and fp8 operands, FGE_F16 with
 * fp16 operands; other pairs yield FGE_ERR_UNSUPPORTED).  FGE_F8E4M3 is the 8-bit format with 4
 * exponent and 3 mantissa bits, bias 7, no infinities (largest value 448, 0x7F / 0xFF are NaN) -
 * the "E4M3" of the OCP 8-bit floating point specification, one byte per element; per-tensor
 * scales go into alpha.  Accumulation and all epilogue arithmetic are fp32;
 * 16-bit stores round to nearest even.  Any M, N, K, batch >= 1 and any
 * strides >= the extents.  Base pointers (X, W, b, out, gamma, beta, aux_out, workspace) must be
 * 16-byte aligned (else FGE_ERR_ALIGN).  The fast kernels move data in 16-byte units: they run
 * when K*sizeof(in), N*sizeof(out), ldx, ldw, ldo and the batch strides are multiples of 16 bytes
 * and a row of X or W is less than 8 MiB from the next
 * (the fused path splits rows of any width over column tiles; a row operation on its own -
 * unfused K3, fge_row_op - spans at most 8192 columns there).  Every other shape is computed too,
 * never refused and never computed wrongly - the paper's benchmark section names silent
 * divisibility assumptions as the typical failure of generated kernels under dynamic shapes:
 * fused_gemm_epilogue copies the operands of a large enough problem (from about 3e7 floating
 * point operations on) into dense buffers in the workspace with K padded by zeros to whole
 * 16-byte units and runs the fast kernels on those (fge_tile_name reports "repacked_operands";
 * when the result's own extents or strides are odd too, it passes through fp32 rows of padded
 * width and an element-granular row kernel); small problems, the stage entry points, the unfused
 * sequence and calls whose workspace only covers it run element-granular kernels (plain fp32 FMA,
 * not tuned; "generic32x32_scalar").  out must not alias X or W.
 */
#ifndef FGE_H
#define FGE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FGE_OK = 0,
    FGE_ERR_NULL = 1,         /* a required pointer is NULL                                  */
    FGE_ERR_BAD_ENUM = 2,     /* act / norm / dtype code or flag bit out of range            */
    FGE_ERR_BAD_SHAPE = 3,    /* M, N, K, batch <= 0, or a stride smaller than the extent    */
    FGE_ERR_UNSUPPORTED = 4,  /* valid request outside the supported set                     */
    FGE_ERR_ALIGN = 5,        /* a base pointer is not 16-byte aligned                       */
    FGE_ERR_WORKSPACE = 6,    /* workspace NULL or smaller than fge_workspace_bytes()        */
    FGE_ERR_HIP = 7           /* a launch failed; see fge_last_hip_error()                   */
} fge_status;

typedef enum { FGE_F32 = 0, FGE_BF16 = 1, FGE_F16 = 2, FGE_F8E4M3 = 3 } fge_dtype;

/* Activations (step A = act(Y)).  GELU_TANH: 0.5 y (1 + tanh(sqrt(2/pi) (y + 0.044715 y^3)));
 * GELU_ERF: 0.5 y (1 + erf(y / sqrt 2)); SILU: y / (1 + exp(-y)); CLAMP: min(max(y, lo), hi). */
typedef enum {
    FGE_ACT_NONE = 0, FGE_ACT_RELU = 1, FGE_ACT_GELU_TANH = 2, FGE_ACT_GELU_ERF = 3,
    FGE_ACT_SILU = 4, FGE_ACT_CLAMP = 5
} fge_act;

/* Row operations over N.
 *   SOFTMAX   : out_j = exp(a_j - m) / sum_l exp(a_l - m),  m = max_j a_j
 *   LAYERNORM : out_j = (a_j - mu) / sqrt(var + eps) * gamma_j + beta_j, biased variance
 *   RMSNORM   : out_j = a_j / sqrt(mean_j(a_j^2) + eps) * gamma_j   (eps inside the root, as in
 *               the paper's RMSNorm sketch, Fig. 2)
 *   LOGSUMEXP : out = A unchanged, aux_out[row] = m + ln sum_j exp(a_j - m)               */
typedef enum {
    FGE_NORM_NONE = 0, FGE_NORM_SOFTMAX = 1, FGE_NORM_LAYERNORM = 2, FGE_NORM_RMSNORM = 3,
    FGE_NORM_LOGSUMEXP = 4
} fge_norm;

/* fge_params.flags.
 *   FGE_FLAG_TWO_PASS : always finish split rows with the second kernel.  Without it the tile
 *   kernel of a large problem finishes its rows itself: the column tiles of a row block run at
 *   the same time, exchange their row statistics through the workspace and wait for each other
 *   (a bounded wait).  That form assumes the launch has the device to itself; set this flag when
 *   several launches may overlap on the device (other streams, other processes).  Before such a
 *   launch the library asks the runtime whether the device holds the whole grid at once; if it
 *   does not, the two-pass form is taken.  A tile whose wait runs out all the same (its row block's
 *   other tiles did not arrive within about 2^20 polls) stores NaN for its rows - and NaN in
 *   aux_out for LOGSUMEXP - and sets the fault word (fge_fault_word_offset): the kernel always
 *   terminates and never stores values normalised with incomplete statistics.  The stage entry
 *   points fge_fused_tiles / fge_fused_finish always take the two-pass form.
 *   FGE_FLAG_IEEE_FP32 : multiply fp32 operands with the fp32 matrix instruction.  Without it
 *   fp32 operands are multiplied on the bf16 matrix instruction after a split of each operand
 *   into two bf16 terms, x = xh + xl:  x*w ~= xl*wh + xh*wl + xh*wh with fp32 accumulation.
 *   Relative error per product <= about 2^-16.5 (a few 1e-5 on the final result, inside the
 *   1e-4 the fp32 path is held to, and exact for operands that bf16 holds exactly) at less than a
 *   fifth of the matrix-pipe time.  bf16 operands are not affected.
 *   FGE_FLAG_NO_SPLIT_K : never cut K into slices.  Without it fused_gemm_epilogue runs a problem
 *   with few tiles and a long K (64x64 tiles, no more of them than compute units, K >= 2048 to
 *   8192 depending on operand type and tile count; see
 *   fge_fused_k_slices) as partial products over 2 to 16 slices of K - one launch, fp32, into the
 *   workspace - which a second kernel adds in slice order (the result does not depend on the
 *   schedule) before scale, bias and activation; a row operation then runs over that fp32
 *   result.  Taken only when the workspace has the room fge_workspace_bytes reports; with a
 *   smaller workspace (or none, where none is needed otherwise) the problem runs unsliced.
 *   FGE_FLAG_TILE(t) : run the tile kernels with tile configuration t (an fge_tile) instead of
 *   the library's own choice - for tuning and tests.  A configuration without kernels for the
 *   operand type (or the narrow-K kernel outside K <= 64, N <= 512, fp32) yields
 *   FGE_ERR_UNSUPPORTED.  Ignored by the gated form and by shapes that take the element-granular
 *   kernels.
 *   FGE_FLAG_NO_TABLE : choose the tile configuration by the library's rule alone.  Without it, for
 *   16-bit and 8-bit operands, the choice first consults a table of the fastest verified
 *   configuration at each point of a sweep over shapes (written by the configuration search of
 *   the Python package on an MI355X) and takes the entry nearest to the problem when one is near.
 *   FGE_FLAG_TEST_EXPIRE_WAIT : for tests of the bounded wait only.  In the one-kernel form the
 *   first column tile of every row block keeps its arrival mark back and every wait gives up
 *   after one poll, so the waits run out while every workgroup still finishes normally; the
 *   affected rows must come back as NaN and the fault word set. */
enum { FGE_FLAG_TWO_PASS = 1, FGE_FLAG_IEEE_FP32 = 2, FGE_FLAG_NO_SPLIT_K = 4, FGE_FLAG_NO_TABLE = 8, FGE_FLAG_TILE_MASK = 0xF00,
       FGE_FLAG_TEST_EXPIRE_WAIT = 0x1000 };
#define FGE_FLAG_TILE(t) ((((int)(t)) + 1) << 8)

/* Tile configurations (rows x columns of one workgroup's output tile).  16-bit and 8-bit
 * operands: 64x64, 64x512, 128x128 (FGE_TILE_128x128_S3, eight waves and three stage buffers,
 * takes its place for problems with at most one such tile per CU), 128x256, 256x128, 256x256;
 * fp32 operands: 64x64, 64x512,
 * 64x128, 128x128 (split product only; on four waves, or on eight - FGE_TILE_128x128_W8 - for
 * problems with one tile per CU) and the persistent narrow-K kernel. */
typedef enum {
    FGE_TILE_64x64 = 0, FGE_TILE_64x512 = 1, FGE_TILE_128x128 = 2, FGE_TILE_256x256 = 3,
    FGE_TILE_NARROW_K = 4, FGE_TILE_64x128 = 5, FGE_TILE_128x256 = 7, FGE_TILE_256x128 = 8,
    FGE_TILE_128x128_W8 = 9, FGE_TILE_128x128_S3 = 10
} fge_tile;

typedef struct fge_params {
    int32_t M, N, K, batch;        /* rows per problem, columns, contraction length, problems  */
    int64_t ldx, ldw, ldo;         /* row strides in elements (K, K, N when dense)             */
    int64_t batch_stride_x;        /* elements between problems in X (M*ldx when dense)        */
    int64_t batch_stride_o;        /* elements between problems in out (M*ldo when dense)      */
    int32_t in_dtype, out_dtype;   /* fge_dtype of X and W / of out and unfused intermediates  */
    float   alpha, post_scale;     /* Y = post_scale * (alpha * X.W^T + b)                     */
    float   clamp_lo, clamp_hi;    /* FGE_ACT_CLAMP bounds                                     */
    float   eps;                   /* LAYERNORM / RMSNORM                                      */
    int32_t flags;                 /* FGE_FLAG_* bits, 0 for the defaults                      */
    const float *gamma, *beta;     /* device, length N; NULL means all ones / all zeros        */
    float  *aux_out;               /* device, batch*M floats; required for LOGSUMEXP only      */
    void   *workspace;             /* device scratch, 16-byte aligned                          */
    size_t  workspace_bytes;       /* its size                                                 */
} fge_params;

/* The fused path (the paper's Section 4.3: a fused operator avoids the intermediate memory
 * accesses and the launches of the composed small operators; chain and row operations as in its
 * Section 3.6 categories and the RMSNorm sketch of Fig. 2): one tile kernel that keeps the
 * accumulators in registers through scale, bias, activation and the in-tile row reduction.  When a row spans several column tiles the
 * tiles publish mergeable row statistics to the workspace; large problems then finish their
 * rows inside the same kernel (see FGE_FLAG_TWO_PASS), others with a light second kernel that
 * merges the statistics and normalises `out` in place.  b may be NULL (no bias). */
int fused_gemm_epilogue(const void *X, const void *W, const float *b, int act, int norm,
                        const fge_params *p, void *out, void *stream);

/* The unfused reference sequence - what the paper's Section 4.3 describes eager execution as:
 * one operator after the other, every intermediate through memory - built from the same device
 * pieces: K1 Y = post_scale*(alpha*
 * X.W^T + b) -> workspace, K2 A = act(Y) -> workspace (-> out for NONE / LOGSUMEXP), K3
 * out = rowop(A).  Intermediates are stored in out_dtype, as an eager framework would. */
int unfused_gemm_epilogue(const void *X, const void *W, const float *b, int act, int norm,
                          const fge_params *p, void *out, void *stream);

/* ---- for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid it): fused_gemm_epilogue with the library's own scratch in
 * place of the caller's workspace.  p->workspace and p->workspace_bytes are ignored; the row
 * statistics of split rows (and, when they fit as well, the partial products of the optional K
 * slices) live in a static device array of FGE_STATIC_SCRATCH_BYTES that is part of the library's
 * code object: every GPU the library runs on holds one copy until the process ends.  The call
 * allocates and frees nothing and, like every other entry point, only enqueues kernels (no memset
 * node; the scratch needs no clearing between calls).  Arguments, results and errors are those of
 * fused_gemm_epilogue, with two additions: a problem whose split-row statistics (or, for shapes
 * on the element-granular kernels, whose fp32 intermediate) exceed the array returns
 * FGE_ERR_WORKSPACE before anything is enqueued - fge_workspace_bytes with FGE_FLAG_NO_SPLIT_K set
 * tells the size in question; and all calls on one GPU share that GPU's array, so two such calls
 * that may overlap on a device (different streams, different threads) race - callers serialise
 * them on one stream.  The device address of the array is asked from the runtime on the first
 * call on each device; fge_static_scratch_init does the same ahead of time for the current
 * device (e.g. before a graph capture starts) and reports a failure as FGE_ERR_HIP. */
enum { FGE_STATIC_SCRATCH_BYTES = 16 << 20 };     /* 16 MiB */
int fused_gemm_epilogue_static(const void *X, const void *W, const float *b, int act, int norm,
                               const fge_params *p, void *out, void *stream);
int fge_static_scratch_init(void);
size_t fge_static_scratch_bytes(void);

/* Device scratch is the caller's (the paper's kernels come with a host wrapper that owns all
 * buffers, Section 3.2, the Coder).  Bytes of workspace the fused (fused != 0) or unfused (fused == 0) path needs for these
 * arguments; 0 is a valid answer.  Returns (size_t)-1 when the arguments are invalid.  The fused
 * figure includes the room for the optional K slices (FGE_FLAG_NO_SPLIT_K); a smaller workspace
 * that still holds the row statistics of split rows is accepted and runs unsliced. */
size_t fge_workspace_bytes(int fused, int act, int norm, const fge_params *p);

/* Where the one-kernel form of split rows reports a wait that ran out: byte offset into the
 * workspace of an int32 that such a launch sets to 1 (it never clears it; the rows of the tiles
 * whose wait ran out are stored as NaN).  (size_t)-1 when fused_gemm_epilogue does not take that
 * form for these arguments.  A caller that wants the check clears the word before the call and
 * reads it after synchronising; a caller that does not will still find the NaN rows. */
size_t fge_fault_word_offset(int act, int norm, const fge_params *p);

/* ---- the gated form (the "SiLU-and-Mul" / "GELU-and-Mul" fused operators of the paper's
 * benchmark section, Section 3.6, followed by the optional row operation):
 *
 *     out = rowop_N( act(post_scale*(alpha*X.W1^T + b1)) * (post_scale*(alpha*X.W2^T + b2)) )
 *
 * W1 and W2 are both N x K with row stride ldw; b1, b2 fp32 of length N or NULL.  Everything
 * else is as for fused_gemm_epilogue.  The fused call runs one tile kernel that forms both
 * products from one staged X panel and applies the gate to the accumulators, for bf16 / fp16 / E4M3
 * operands in shapes the fast kernels take; every other case (fp32 operands, odd extents) runs
 * the unfused sequence: two GEMMs into the workspace (fp32 operands always on the fp32 matrix
 * instruction here: the gate multiplies two products and their errors), the gate as an
 * elementwise kernel, the row operation.  A small problem with a long K (at most 96 of the gated
 * kernel's 256 x 128 tiles, K >= 1024) runs as fp32 partial products of both GEMMs instead (K cut
 * into slices where fused_gemm_epilogue would cut it), one kernel that adds the slices and
 * applies scale, bias, activation and gate, and the row operation on that fp32 result - when
 * the workspace has the room, else the tile kernel.  fge_gated_workspace_bytes gives the
 * workspace either call needs; fge_gated_tile_name names what the fused call runs
 * ("partial_products_then_gate" for small problems, "unfused_sequence" for the fallback). */
int fused_gated_gemm_epilogue(const void *X, const void *W1, const void *W2, const float *b1,
                              const float *b2, int act, int norm, const fge_params *p, void *out,
                              void *stream);
int unfused_gated_gemm_epilogue(const void *X, const void *W1, const void *W2, const float *b1,
                                const float *b2, int act, int norm, const fge_params *p, void *out,
                                void *stream);
size_t fge_gated_workspace_bytes(int fused, int act, int norm, const fge_params *p);
const char *fge_gated_tile_name(int act, int norm, const fge_params *p);

/* ---- the individual stages, callable on their own (the two paths above are built from them) */

/* Fused stage 1: the tile kernel, always in the two-pass form.  When the chosen tile spans N it
 * produces the final out; otherwise the tiles park their values in out and publish per-strip row
 * statistics to the workspace (split rows, paper Fig. 2: statistics first, normalise second). */
int fge_fused_tiles(const void *X, const void *W, const float *b, int act, int norm,
                    const fge_params *p, void *out, void *stream);
/* Fused stage 2: merge per-tile row statistics from the workspace and finish `out` in place.
 * A no-op (FGE_OK, nothing enqueued) when stage 1 already produced the final result. */
int fge_fused_finish(int act, int norm, const fge_params *p, void *out, void *stream);
/* 1 if fge_fused_finish has work to do for these arguments, 0 if not, negative on bad args.
 * Depends on the arguments only (not on the stream or the device). */
int fge_fused_needs_finish(int act, int norm, const fge_params *p);
/* Slices of K that fused_gemm_epilogue cuts these arguments into when the workspace has the
 * room (1: none; see FGE_FLAG_NO_SPLIT_K), negative on bad args.  The stage entry points
 * fge_fused_tiles / fge_fused_finish never slice. */
int fge_fused_k_slices(int act, int norm, const fge_params *p);

/* Unfused K1: Y (rows x N, out_dtype, row stride ldo) = post_scale * (alpha * X.W^T + b). */
int fge_gemm_bias(const void *X, const void *W, const float *b, const fge_params *p,
                  void *Y, void *stream);
/* Unfused K2: A = act(Y), both rows x N in out_dtype with row stride ldo; A may equal Y. */
int fge_activation(const void *Y, int act, const fge_params *p, void *A, void *stream);
/* Unfused K3: out = rowop(A), both rows x N in out_dtype with row stride ldo; out may equal A. */
int fge_row_op(const void *A, int norm, const fge_params *p, void *out, void *stream);

/* Static description of a status code (every refusal is explicit: the paper's Section 3.6 counts
 * a silently wrong result as the failure, not an error return). */
const char *fge_status_string(int status);
/* hipError_t (as int) recorded by the calling thread's last FGE_ERR_HIP, else 0. */
int fge_last_hip_error(void);
/* Name of the tile configuration the fused path picks for these arguments (static string,
 * e.g. "256x256_w2x4"); NULL on invalid arguments.  For reports and tests. */
const char *fge_tile_name(int fused, int act, int norm, const fge_params *p);

#ifdef __cplusplus
}
#endif
#endif /* FGE_H */
