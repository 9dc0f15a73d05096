/*
 * esparse.h - C ABI of the MI355X (gfx950) implementation of the E-Sparse hot path
 * (E-Sparse: entropy-based N:M sparsity for LLMs, arXiv 2310.15929).
 *
 * Three offline / online stages of one linear layer  Y[M,N] = X[M,K] . W[N,K]^T :
 *   esparse_prune     calibration features + weights -> channel permutation + n:m mask
 *                     (Section 3.2 eq. 1-3, Section 3.3, Algorithm 1)
 *   esparse_compress  masked weights -> kept values + 2-bit in-group indices (Section 4, step 1)
 *   esparse_spmm      activations x compressed weights -> output, on sparse MFMA (Section 4)
 * plus the dense GEMM of the same shapes (the "Dense GEMM" column of Table 5), the per-shape
 * choice of the fastest kernel variant (Section 4, step 2) and size queries.
 *
 * Conventions
 *   - Notation: n:m = keep n_keep of every m_group consecutive RE-ORDERED input channels of each
 *     output row.  theta ("perm") is a gather permutation: re-ordered position p holds original
 *     channel perm[p]; W' = W[:, perm], X' = X[:, perm].
 *   - Unless a parameter is marked HOST, every data pointer is a DEVICE pointer owned by the
 *     caller, row-major, contiguous and 16-byte aligned.  The library never frees or keeps them.
 *   - All GPU work is enqueued on the context's stream.  esparse_spmm, esparse_dense_gemm,
 *     esparse_dense_pack, esparse_stage_activations and the *_staged products do not synchronise; esparse_prune,
 *     esparse_compress, esparse_channel_stats and esparse_tune do (they return host results).
 *   - Every function returns an esparse_status (0 = ok, negative = error) and never throws.
 *     Arguments are validated before the first GPU call; on an argument error nothing is
 *     launched and outputs are untouched.  esparse_last_error gives a message.
 *   - Calibration features and activations must be finite.
 */
#ifndef ESPARSE_H
#define ESPARSE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct esparse_ctx esparse_ctx; /* opaque: device, stream, scratch, last error */

typedef enum { ESPARSE_F16 = 0, ESPARSE_BF16 = 1 } esparse_dtype;

typedef enum {
  ESPARSE_OK = 0,
  ESPARSE_EINVAL = -1,       /* null pointer, bad size, misaligned pointer                     */
  ESPARSE_EUNSUPPORTED = -2, /* pattern / dtype / size the library has no kernel for            */
  ESPARSE_ENOMEM = -3,       /* internal scratch allocation failed                              */
  ESPARSE_EHIP = -4,         /* a HIP call failed (message has the HIP error string)            */
  ESPARSE_EBADMASK = -5,     /* a group of the mask does not keep exactly n_keep                */
  ESPARSE_EBADPERM = -6,     /* perm is not a bijection on [0, K)                               */
  ESPARSE_EWORKSPACE = -7    /* caller workspace smaller than esparse_spmm_workspace reports    */
} esparse_status;

/* Switches of esparse_prune_opts.flags: the four rows of the ablation of Table 4. */
#define ESPARSE_USE_ENTROPY 1u /* IR_c term of eq. 3            */
#define ESPARSE_USE_NORM 2u    /* alpha * AM_c term of eq. 3    */
#define ESPARSE_USE_GNS 4u     /* global naive shuffle          */
#define ESPARSE_USE_LBS 8u     /* local block shuffle           */
#define ESPARSE_USE_ALL 15u

typedef struct {
  int n_keep, m_group;  /* 2:4 or 4:8                                                          */
  int block;            /* local-block-shuffle block size in channels (paper default 256);     */
                        /* multiple of m_group, divides K, <= 256                              */
  int bins;             /* histogram bins of eq. 1 (paper: 100); 1..256                        */
  double alpha;         /* weight of the norm term in eq. 3 (the paper prints no value)        */
  unsigned flags;       /* ESPARSE_USE_*                                                       */
  long long max_swaps;  /* cap on exchanges per block; 0 = until none improves (Algorithm 1)   */
} esparse_prune_opts;

/* ---- context -------------------------------------------------------------------------------
 * esparse_create binds a context to HIP device `device` and to `hip_stream` (a hipStream_t passed
 * as void*, NULL = the default stream).  Contexts are not thread-safe; use one per thread. */
int esparse_create(esparse_ctx** out, int device, void* hip_stream);
void esparse_destroy(esparse_ctx* ctx);
int esparse_set_stream(esparse_ctx* ctx, void* hip_stream);
const char* esparse_last_error(const esparse_ctx* ctx); /* HOST string owned by the context */
const char* esparse_version(void);

/* ---- Section 3.2, eq. 1-2: per-channel statistics of the calibration features ---------------
 * calib[T,K] (dtype) -> entropy IR_c over `bins` equal-width bins spanning the channel's own
 * [min, max] (natural log, top edge closed), amplitude AM_c = ||X_c||_2 (sum of squares exact,
 * rounded once).  ir_out / am_out: HOST double[K], either may be NULL.  Synchronises. */
int esparse_channel_stats(esparse_ctx* ctx, const void* calib, long long T, long long K,
                          esparse_dtype dtype, int bins, double* ir_out, double* am_out);

/* ---- Section 3.2 eq. 3 + Section 3.3 + Algorithm 1: metric, channel shuffle, n:m mask -------
 * calib[T,K], W[N,K] (dtype) -> perm_out[K] int32 (DEVICE), mask_out[N,K] uint8 (DEVICE, one byte
 * per weight, 1 = kept, in RE-ORDERED channel order).  Optional HOST outputs (NULL to skip):
 * score_out double[K] (s_c = IR_c + alpha AM_c), swaps_out int64[K/block] (exchanges made per
 * block), retained_out double[1] (objective of eq. 5: total metric kept).
 * Ties: equal metric -> lower position kept; equal channel means -> lower channel first; equal
 * improvements -> smallest (i, j).  Synchronises and allocates internal scratch. */
int esparse_prune(esparse_ctx* ctx, const void* calib, long long T, const void* W, long long N,
                  long long K, esparse_dtype dtype, const esparse_prune_opts* opts,
                  int32_t* perm_out, uint8_t* mask_out, double* score_out, int64_t* swaps_out,
                  double* retained_out);

/* Same as esparse_prune from the shuffle on, with the channel scores s_c given (HOST double[K]). */
int esparse_prune_with_scores(esparse_ctx* ctx, const double* score, const void* W, long long N,
                              long long K, esparse_dtype dtype, const esparse_prune_opts* opts,
                              int32_t* perm_out, uint8_t* mask_out, int64_t* swaps_out,
                              double* retained_out);

/* ---- Section 4, step 1: compressed format ---------------------------------------------------
 * Sizes (closed form; 2 bits of index per kept value -> 56.25 % of dense 16-bit for n/m = 1/2):
 *   values_bytes = N*K*n/m * 2,  meta_bytes = N*K/8,
 *   native_bytes = 1.125 * Np * Kp with Np = N rounded up to 16, Kp = K rounded up to 256
 *                  (2:4 and 4:8 alike: 1 byte of kept values + 1 bit of metadata per weight).
 * Any of the three outputs may be NULL. */
int esparse_compressed_size(long long N, long long K, int n_keep, int m_group, esparse_dtype dtype,
                            size_t* values_bytes, size_t* meta_bytes, size_t* native_bytes);

/* W[N,K] in ORIGINAL channel order, mask[N,K] uint8 in re-ordered order (NULL = keep the non-zero
 * weights; a group with fewer than n non-zeros is topped up with its lowest-position zeros),
 * perm[K] int32 (NULL = identity).  Outputs, each optional (NULL to skip):
 *   values_out [N, K*n/m] dtype : kept W[j, perm[p]] in ascending p
 *   meta_out   2:4 -> uint32[N, ceil(K/32)]: field f (f-th kept value of the row) = its position in
 *              its group of 4, at bit 2*(f mod 16) of word f div 16;
 *              4:8 -> uint8[N, K/8]: occupancy bitmap of each group of 8
 *   native_out the same data in the order the SpMM kernels stream it, zero padded.
 *              2:4: unit = (row, 16 re-ordered channels) = 8 kept values (16 B) + one uint16 of
 *              indices; values units ordered [row/16][chunk/4][chunk%4][row%16], then at byte
 *              offset Np*Kp the uint16 units ordered [row/16][chunk/16][chunk%4][row%16][(chunk/4)%4].
 *              4:8: the group of row 16 rt + r covering re-ordered channels 64 ks + 32 h + 8 g .. + 8
 *              belongs to lane 16 g + r: its 4 kept values are half h (8 B) of the 16-byte unit
 *              (rt * Kp/64 + ks) * 64 + lane, its pattern code byte h of the uint16 unit at the place the
 *              2:4 form keeps that lane's indices for step ks.  Pattern code = the index of the group's
 *              occupancy bitmap among the 70 bitmaps with four bits set, in ascending order (0x0f -> 0,
 *              0x17 -> 1, ..., 0xf0 -> 69); padding groups hold zero values and code 0.
 * Errors: EBADMASK (a group keeping != n, or > n non-zeros with mask NULL), EBADPERM.
 * Synchronises (it reports those two errors). */
int esparse_compress(esparse_ctx* ctx, const void* W, const uint8_t* mask, const int32_t* perm,
                     long long N, long long K, esparse_dtype dtype, int n_keep, int m_group,
                     void* values_out, void* meta_out, void* native_out);

/* ---- Section 4: sparse product ---------------------------------------------------------------
 * Y[M,N] (dtype) = X[:, perm] . W'_sparse^T with fp32 accumulation; X[M,K] is in ORIGINAL channel
 * order, the re-ordering of Section 3.3 is applied while X is staged.  native_w from
 * esparse_compress.  workspace: DEVICE scratch of at least esparse_spmm_workspace bytes,
 * 256-byte aligned; it is overwritten.  variant: -1 = the one chosen by esparse_tune for this shape
 * (a built-in rule if never tuned), >= 0 = a specific kernel variant (EINVAL if out of range).
 * esparse_spmm_workspace (host only, no context): variant -1 = the size that serves every variant of the
 * shape - what a call with variant -1 requires, since tuning may change the choice after the caller has
 * allocated; variant >= 0 = what that variant needs (the staged activations, plus fp32 partial tiles only
 * for variants that split K over workgroups) - what a call naming that variant requires.
 * M = 0 is a no-op.  n:m = 2:4 runs on the sparse matrix instruction.  n:m = 4:8 (Section 4 lists it as a
 * format the hardware of the paper cannot multiply; there is no instruction for it here either): the
 * kernels expand each group to a dense operand in registers (byte-permute selectors looked up by the
 * group's pattern code) and use the dense instruction, which pays where the product is bound by reading
 * the weights; at prefill sizes (the tile48 variants, 64 tokens and more; the default beyond 128) it runs
 * at 0.7-0.9 of the dense product's speed on 56 % of its weight bytes.  Only decode-kernel variants
 * (inputs longer than 64 tokens: 64 at a time), the stream variants with a ring of four slots (at most
 * 128 tokens) and the tile48 variants apply (EUNSUPPORTED for the others).  Other n:m: EUNSUPPORTED.
 * Does not synchronise. */
int esparse_spmm_workspace(long long M, long long N, long long K, int variant, size_t* bytes);
int esparse_spmm(esparse_ctx* ctx, const void* X, long long M, const void* native_w,
                 const int32_t* perm, long long N, long long K, esparse_dtype dtype, int n_keep,
                 int m_group, void* Y, void* workspace, size_t workspace_bytes, int variant);
/* esparse_spmm for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same product, same kernels and bitwise the same
 * result as esparse_spmm with the same variant; the scratch (staged activations, partial tiles of the variants
 * that split K) is a fixed array of ESPARSE_STATIC_SCRATCH_BYTES in the library's device image, one per GPU,
 * held until the process ends.  The call allocates and frees nothing on the device.  variant -1: where the tuned
 * (or built-in) choice keeps fp32 partial tiles that do not fit the array, the built-in choice among the kernels
 * without partial tiles runs instead (a decode kernel up to 64 tokens, tile32_w8_t128 up to 128, tile32_w8_t256
 * beyond; 4:8: tile48_w8_r128_t256).  A shape whose variant still needs more scratch than the array holds is
 * rejected with ESPARSE_EWORKSPACE and nothing is launched (the message gives both sizes); the first call on a GPU looks the array's device address up (that GPU current).  Every call on one GPU
 * uses the same array, on whatever stream its context has: calls that overlap on one GPU race - order them on
 * one stream or with events.  No part of the array needs clearing between calls (each kernel reads only what an
 * earlier kernel of the same call wrote).  Other errors as esparse_spmm.  Does not synchronise. */
#define ESPARSE_STATIC_SCRATCH_BYTES (64u << 20)
int esparse_spmm_static(esparse_ctx* ctx, const void* X, long long M, const void* native_w,
                        const int32_t* perm, long long N, long long K, esparse_dtype dtype, int n_keep,
                        int m_group, void* Y, int variant);
/* The two halves of esparse_spmm as separate calls, for callers that multiply one activation
 * matrix with several weight matrices sharing one perm, or that time the multiply alone:
 * esparse_stage_activations writes X[:, perm] in the kernels' operand order into the workspace
 * (sized by esparse_spmm_workspace(M, N, K) for the largest N that will use it);
 * esparse_spmm_staged multiplies what the workspace holds.  Same errors as esparse_spmm. */
int esparse_stage_activations(esparse_ctx* ctx, const void* X, long long M, const int32_t* perm,
                              long long N, long long K, esparse_dtype dtype, void* workspace,
                              size_t workspace_bytes);
int esparse_spmm_staged(esparse_ctx* ctx, long long M, const void* native_w, long long N, long long K,
                        esparse_dtype dtype, int n_keep, int m_group, void* Y, void* workspace,
                        size_t workspace_bytes, int variant);
int esparse_spmm_num_variants(void);
const char* esparse_spmm_variant_name(int variant);

/* ---- Table 5, "Dense GEMM" column: the dense product on the same shapes ----------------------
 * esparse_dense_pack re-tiles W[N,K] into the order the dense kernel streams (packed_out:
 * esparse_dense_packed_size bytes = 2 * Np * Kp, rows padded to 16, K to 256, zero filled).
 * esparse_dense_gemm: Y[M,N] = X . W^T, same workspace query as the sparse product. */
int esparse_dense_packed_size(long long N, long long K, size_t* bytes);
int esparse_dense_pack(esparse_ctx* ctx, const void* W, long long N, long long K,
                       esparse_dtype dtype, void* packed_out);
int esparse_dense_gemm(esparse_ctx* ctx, const void* X, long long M, const void* packed_w,
                       long long N, long long K, esparse_dtype dtype, void* Y, void* workspace,
                       size_t workspace_bytes, int variant);

int esparse_dense_gemm_staged(esparse_ctx* ctx, long long M, const void* packed_w, long long N,
                              long long K, esparse_dtype dtype, void* Y, void* workspace,
                              size_t workspace_bytes, int variant);

/* ---- Section 4 / Table 5 (decoder): several products of one shape in one call ---------------------
 * At decode sizes one product of a 4096 x 4096 matrix is a few microseconds of kernel, mostly launch and
 * ramp-up; the linear layers that read the same hidden state (q/k/v, gate/up) have the same shape.  This
 * call runs count (1..4) products Y[i] = X[i][:, perm[i]] . W'_i^T, all with the same M, N, K, dtype
 * and n:m, through one staging launch and one multiply launch when a decode kernel serves the shape
 * (the default up to 32 tokens), and one after the other otherwise.  X, native_w, perm, Y: HOST arrays of count
 * DEVICE pointers (perm may be NULL = identity for all, or hold NULL entries); members may share X.
 * workspace: DEVICE, 256-byte aligned, at least esparse_spmm_group_workspace bytes.  Results are
 * bitwise those of esparse_spmm with the same variant.  Errors as esparse_spmm; count outside 1..4:
 * EINVAL.  Does not synchronise. */
int esparse_spmm_group_workspace(int count, long long M, long long N, long long K, size_t* bytes);
int esparse_spmm_group(esparse_ctx* ctx, int count, const void* const* X, long long M,
                       const void* const* native_w, const int32_t* const* perm, long long N, long long K,
                       esparse_dtype dtype, int n_keep, int m_group, void* const* Y, void* workspace,
                       size_t workspace_bytes, int variant);

/* The two halves of esparse_spmm_group (for callers that time the multiply alone); they exist where a
 * decode kernel serves the shape (EUNSUPPORTED otherwise).  n_keep / m_group and variant must be the
 * ones of the multiply that follows. */
int esparse_stage_activations_group(esparse_ctx* ctx, int count, const void* const* X, long long M,
                                    const int32_t* const* perm, long long N, long long K,
                                    esparse_dtype dtype, int n_keep, int m_group, void* workspace,
                                    size_t workspace_bytes, int variant);
int esparse_spmm_group_staged(esparse_ctx* ctx, int count, long long M, const void* const* native_w,
                              long long N, long long K, esparse_dtype dtype, int n_keep, int m_group,
                              void* const* Y, void* workspace, size_t workspace_bytes, int variant);

/* The dense counterpart (speedup denominator of the grouped call): count products
 * Y[i] = X[i] . W_i^T with packed_w[i] from esparse_dense_pack.  Same conventions and workspace size. */
int esparse_dense_gemm_group(esparse_ctx* ctx, int count, const void* const* X, long long M,
                             const void* const* packed_w, long long N, long long K, esparse_dtype dtype,
                             void* const* Y, void* workspace, size_t workspace_bytes, int variant);

/* ---- Section 4, step 2: pick and remember the fastest variant for a shape --------------------
 * Times every applicable variant of esparse_spmm (sparse = 1: 2:4, sparse = 2: 4:8) or esparse_dense_gemm (sparse = 0) on
 * scratch operands (finite pseudo-random values) of shape (M, N, K) and stores the winner in the context; later
 * calls with variant = -1 use it.  The timed launches rotate over copies of the weight operand
 * (about 640 MiB of them, at least two), so that the weights come from HBM as they do when a
 * model reads each matrix once per step.  best_variant (HOST, optional) receives its id.  The table can be
 * saved to / restored from a text file (HOST path).  Synchronises; allocates scratch. */
int esparse_tune(esparse_ctx* ctx, long long M, long long N, long long K, esparse_dtype dtype,
                 int sparse, int* best_variant, float* best_ms);
/* The same search for launches of `count` products of one shape (esparse_spmm_group, esparse_dense_gemm_group; count in
 * 1..4): a group fills the chip differently from a single product, so its fastest variant can differ.  Group calls with
 * variant = -1 use the choice tuned for their count, else the one tuned for the single product, else the default.
 * In the text file a line may end in the count. */
int esparse_tune_group(esparse_ctx* ctx, int count, long long M, long long N, long long K, esparse_dtype dtype,
                       int sparse, int* best_variant, float* best_ms);
int esparse_tune_save(const esparse_ctx* ctx, const char* path);
int esparse_tune_load(esparse_ctx* ctx, const char* path);

/* ---- Section 3.3, eq. (4): output error of a pruned layer -------------------------------------
 * Yref, Y (DEVICE, row-major [M, N], dtype): two outputs of the same activations, normally
 * esparse_dense_gemm with the unpruned weights and esparse_spmm with the pruned ones.  Writes
 * (HOST doubles) err_num = || Yref - Y ||_F^2 and err_den = || Yref ||_F^2, accumulated in float64 in
 * a fixed order (deterministic); eq. (4)'s objective is err_num, its relative form err_num / err_den.
 * Synchronises the context's stream; allocates a small scratch buffer.  M * N == 0 gives 0, 0.
 * Errors: ESPARSE_EINVAL (null pointer, negative size, bad dtype), ESPARSE_ENOMEM, ESPARSE_EHIP. */
int esparse_output_error(esparse_ctx* ctx, const void* Yref, const void* Y, long long M, long long N,
                         esparse_dtype dtype, double* err_num, double* err_den);

/* ---- Measurement aid: what the matrix pipes sustain on this chip -------------------------------
 * Not a step of the method: the ceiling its product kernels (Section 4) are compared with, beside the published
 * peak.  One workgroup of 8 waves per compute unit issues the matrix instruction of the tile kernels back to back for
 * about 40 ms; *tflops (HOST) receives the rate in effective TFLOP/s: 2 x 32 x 32 x 32 flops per 2:4 instruction
 * (sparse = 1, v_smfmac_f32_32x32x32), 2 x 32 x 32 x 16 per dense one (sparse = 0, v_mfma_f32_32x32x16), fp16 or bf16.
 * random_operands = 1: values with random signs and mantissas, the case of real data; 0: zeros, on which the chip holds
 * a higher clock.  mix = 0: operands held in registers (no LDS, no memory traffic).  mix = 1 / 2 (2:4 on random
 * operands only, else EUNSUPPORTED): per 16 multiplies - one 64-channel stage of the 8-wave prefill kernel - also that
 * stage's operand reads out of LDS (1), and the DMA of a coming stage's operands from an L2-resident region of global
 * memory into LDS with the stage's counted wait and barrier (2): what the kernel's instruction mix reaches when
 * nothing waits for data.  Synchronises the context's stream; allocates small scratch buffers.
 * Errors: ESPARSE_EINVAL (null pointer, sparse / random_operands not 0 / 1, mix outside 0..2), ESPARSE_EUNSUPPORTED
 * (dtype, mix), ESPARSE_ENOMEM, ESPARSE_EHIP. */
int esparse_matrix_rate(esparse_ctx* ctx, int sparse, esparse_dtype dtype, int random_operands, int mix, double* tflops);

/* The same for the memory system: *gbs (HOST) receives the rate, in GB/s, of a plain streaming read of `bytes` bytes
 * per launch (16 bytes per lane, one workgroup of 1024 threads per compute unit), averaged over 24 launches that walk through a buffer larger
 * than the last-level cache, so that every launch reads from HBM.  The decode kernels (Section 4, Table 5 decoder rows)
 * read 1.125 N K bytes per launch and cannot be faster than this for their size: launch, ramp-up and drain are a fixed
 * few microseconds.  Synchronises the context's stream; allocates max(2 bytes, 640 MiB) of scratch.
 * Errors: ESPARSE_EINVAL (null pointer, bytes outside 4 KiB .. 8 GiB), ESPARSE_ENOMEM, ESPARSE_EHIP. */
int esparse_read_rate(esparse_ctx* ctx, size_t bytes, double* gbs);

#ifdef __cplusplus
}
#endif
#endif /* ESPARSE_H */
