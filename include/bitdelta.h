/* bitdelta.h - C ABI of the MI355X (gfx950) BitDelta library.
 *
 * The library implements the data-parallel hot path of BitDelta (arxiv 2402.10193):
 *   - the offline compressor of Sec. 3.1:  Delta = W_fine - W_base, sign bits (Eq. 1-2),
 *     alpha = mean |Delta| (Eq. 4);
 *   - the multi-tenant serving linear of Sec. 3.3, Eq. 6:
 *         y_t = x_t . W_base^T + alpha_{tenant(t)} * ( x_t . Sign(Delta_{tenant(t)})^T )
 *     for a batch of tokens that share one fp16 base matrix while each token uses the
 *     1-bit delta of its own tenant (the batched W_INT1 A_FP16 product of Sec. 4.3).
 *
 * Conventions shared by every entry point
 *   - Plain C, no exceptions.  Every call returns a bd_status; BD_OK is 0.
 *   - Unless a parameter says HOST, pointers are DEVICE pointers owned by the caller.  The
 *     library never allocates or frees device memory and keeps no state between calls (one
 *     exception, stated there: bd_compress_noalloc uses a fixed array inside the library).
 *   - fp16 tensors are passed as uint16_t bit patterns (IEEE binary16).
 *   - A weight matrix is [out, in] row-major: `in` (the reduction dimension) is contiguous.
 *     `in` must be a multiple of 32, otherwise BD_ERR_SHAPE.
 *   - Packed signs are uint32_t [out, in/32] row-major.  Bit j (least significant first) of
 *     word w in row n is the sign of element k = 32*w + j:  1 means +1 (Delta > 0),
 *     0 means -1 (Delta <= 0, so a zero delta is -1 as in Eq. 2; NaN also packs as 0).
 *   - Tensor pointers must be 16-byte aligned (BD_ERR_ALIGN); rows are then aligned too.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work; they never synchronise.  Argument checks run on the host before anything
 *     is enqueued, so a call that returns an error has launched nothing.
 *   - Scratch memory comes from the caller: `workspace` must hold at least
 *     bd_workspace_bytes(op, ...) bytes and be 256-byte aligned (BD_ERR_WORKSPACE otherwise).
 *     It may be reused by the next call on the same stream.
 *   - Results are deterministic: no floating-point atomics; the same inputs give the same bits.
 */
#ifndef BITDELTA_H
#define BITDELTA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum bd_status {
    BD_OK = 0,
    BD_ERR_NULL = 1,        /* a required pointer is NULL */
    BD_ERR_SHAPE = 2,       /* negative size, in % 32 != 0, or a size beyond the supported range */
    BD_ERR_ALIGN = 3,       /* a tensor pointer is not 16-byte aligned */
    BD_ERR_TENANT = 4,      /* a tenant id is outside [0, n_tenants) */
    BD_ERR_WORKSPACE = 5,   /* workspace missing, too small or misaligned */
    BD_ERR_DEVICE = 6,      /* the HIP runtime reported an error when enqueuing */
    BD_ERR_UNSUPPORTED = 7, /* unknown kernel variant, or one that cannot run these sizes */
    BD_ERR_ALIAS = 8,       /* an output range overlaps an input range */
    BD_ERR_FORMAT = 9,      /* a delta image is malformed (magic, sizes, offsets, checksum) */
    BD_ERR_IO = 10,         /* a file could not be opened, read or written */
    BD_ERR_TOO_LARGE = 11   /* a size beyond the fixed limit of an entry point that brings its own scratch */
} bd_status;

typedef enum bd_op {
    BD_OP_PACK_SIGNS = 0,
    BD_OP_COMPRESS = 1,
    BD_OP_LINEAR_MULTITENANT = 2,
    BD_OP_LINEAR_GEMM = 3,           /* bd_linear_multitenant_gemm_kbit / _gemm_q8: the token tables, any T >= 1 */
    BD_OP_LINEAR_TILED_GEMM = 4      /* bd_linear_multitenant_tiled_gemm: token tables and the tenants' pointer table */
} bd_op;

/* Text for a status code (static storage, never NULL). */
const char* bd_status_string(bd_status s);

/* Library version: major*10000 + minor*100 + patch. */
int bd_version(void);

/* Bytes of workspace the given op needs for these sizes (0 if none).  Sizes that the op
 * would reject give 0. */
size_t bd_workspace_bytes(bd_op op, int64_t T, int64_t out, int64_t in, int32_t n_tenants);

/* Eq. 2 applied to an explicit delta matrix.
 *   delta_f16 [out, in] fp16  ->  packed [out, in/32].
 * out == 0 or in == 0 is a no-op returning BD_OK. */
bd_status bd_pack_signs(const uint16_t* delta_f16, int64_t out, int64_t in,
                        uint32_t* packed, void* stream);

/* The 1-bit quantiser of Sec. 3.1 for one matrix of one fine-tune.
 *   Delta = f32(w_ft) - f32(w_base)                          (IEEE binary32)
 *   packed <- sign bits of Delta                             (Eq. 2; equals w_ft > w_base)
 *   *alpha <- fp16_rne( sum |Delta| / (out*in) ) as a float  (Eq. 4; the sum runs in binary64)
 * w_base_f16, w_ft_f16: [out, in]; packed: [out, in/32]; alpha: one float on the device.
 * Inf/NaN in the inputs propagate into alpha; they are not errors.
 * out == 0 or in == 0: packed untouched, *alpha <- 0. */
bd_status bd_compress(const uint16_t* w_base_f16, const uint16_t* w_ft_f16,
                      int64_t out, int64_t in,
                      uint32_t* packed, float* alpha,
                      void* workspace, size_t workspace_bytes, void* stream);

/* bd_compress for callers that cannot allocate device memory or carry a workspace around: code under HIP graph
 * capture, tight serving loops that compress an incoming fine-tune between decode steps, harnesses that forbid
 * hipMalloc.  Same kernels, same arithmetic and the same bits in packed and *alpha as bd_compress; the partial sums
 * of Eq. 4 go to an array inside the library instead (16 KiB of device memory per GPU the library runs on, held until
 * the process ends; its address is looked up on the first call on each device).  The call allocates and frees nothing.
 *   out * in <= BD_COMPRESS_NOALLOC_MAX_ELEMENTS, else BD_ERR_TOO_LARGE (nothing launched); other errors as
 *   bd_compress.
 * All calls on one GPU share that array: two of them may not overlap in time (different streams without an
 * ordering between them race; calls on one stream are ordered and safe).  Nothing in the array has to be
 * cleared between calls: every slot that is read has been written by the same call before. */
#define BD_COMPRESS_NOALLOC_MAX_ELEMENTS ((int64_t)1 << 32)
bd_status bd_compress_noalloc(const uint16_t* w_base_f16, const uint16_t* w_ft_f16,
                              int64_t out, int64_t in,
                              uint32_t* packed, float* alpha, void* stream);

/* bd_compress for n matrices (say, the linears of one layer of one fine-tune) in two launches instead of
 * 2 n: same arithmetic, and matrix m is cut into blocks exactly as bd_compress would cut it, so packed[m] and
 * alpha[m] are bit for bit what n separate calls give.
 *   w_base_f16, w_ft_f16, packed, out, in   HOST arrays of n entries (the pointers in them: device memory)
 *   alpha                                   device array of n floats
 *   workspace                               BD_COMPRESS_BATCH_MAX * bd_workspace_bytes(BD_OP_COMPRESS, ...) bytes
 * More than BD_COMPRESS_BATCH_MAX matrices run as several such pairs of launches.  Errors as bd_compress;
 * no packed[m] may overlap any input matrix or another packed[o] (BD_ERR_ALIAS). */
#define BD_COMPRESS_BATCH_MAX 8
bd_status bd_compress_batch(int32_t n, const uint16_t* const* w_base_f16, const uint16_t* const* w_ft_f16,
                            const int64_t* out, const int64_t* in, uint32_t* const* packed, float* alpha,
                            void* workspace, size_t workspace_bytes, void* stream);

/* The multi-tenant linear of Eq. 6.
 *   x_f16            [T, in]   fp16 activations, one row per token
 *   w_base_f16       [out, in] fp16 base weight shared by every token
 *   packed_by_tenant device array of n_tenants device pointers, each [out, in/32]
 *   alpha_by_tenant  device array of n_tenants floats
 *   tenant_of_token  HOST array of T ints in [0, n_tenants): which delta each token uses.
 *                    Any order, repeats allowed; tokens of one tenant are grouped inside the
 *                    call so that each delta is streamed once.  A tenant without a token costs
 *                    nothing.
 *   y_f16            [T, out]  fp16 result; must not overlap x or w_base (BD_ERR_ALIAS)
 * Both products accumulate in binary32, alpha multiplies the finished +-1 sum in binary32 and
 * the result is rounded once to fp16 (nearest even).
 * T == 0 or out == 0 is a no-op returning BD_OK.  T up to 65535.
 * Up to 32 tokens run as one decode launch and need no workspace.  More tokens (the prefill regime
 * of Sec. 4.3: many tokens per tenant) can run as ONE matrix-core GEMM launch over all tokens if
 * `workspace` holds bd_workspace_bytes(BD_OP_LINEAR_MULTITENANT, T, out, in, n_tenants) bytes
 * (256-byte aligned; it receives the token permutation).  With a NULL or smaller workspace the same
 * result is produced by ceil(T / 32) decode launches, each re-reading the base; with a workspace the
 * library takes whichever of the two a cost estimate on the host says is quicker (GEMM tiles hold one
 * tenant's tokens only, so a batch with a few tokens per tenant is cheaper as decode launches).
 * Speed: this call reads the tensors in the canonical row-major layout, which costs a decode launch four times the
 * cache accesses per byte of the serving layout; a decode step through it runs at about two thirds of the rate of
 * bd_linear_multitenant_tiled on the same matrices (and the grouped tiled call saves three launches per layer on top).
 * A server re-tiles once (bd_tile_base, bd_tile_signs) and decodes through the tiled calls; this call is the one that
 * needs no preparation. */
bd_status bd_linear_multitenant(const uint16_t* x_f16, const uint16_t* w_base_f16,
                                const uint32_t* const* packed_by_tenant,
                                const float* alpha_by_tenant,
                                const int32_t* tenant_of_token,
                                uint16_t* y_f16,
                                int64_t T, int64_t out, int64_t in, int32_t n_tenants,
                                void* workspace, size_t workspace_bytes, void* stream);

/* Same operation with the kernel chosen by the caller instead of by the library; meant for
 * benchmarking the kernel variants against each other.
 *   variant 0  library's choice (identical to bd_linear_multitenant)
 *   variant 1  plain vector-ALU kernel: one wavefront per output row, DPP reductions
 *   variant 2  the matrix-core decode kernel of the serving path reading the row-major tensors as they are
 *              (in % 128 == 0 and a base below 4 GiB, else BD_ERR_UNSUPPORTED); the library's choice for such sizes
 *   variant 4, 5, 6  the prefill GEMM with 128 x 128 tiles / 128 x 256 tiles and 4 wavefronts / 128 x 256
 *              tiles and 8 wavefronts (T > 32 and a workspace as for variant 0, else BD_ERR_UNSUPPORTED /
 *              BD_ERR_WORKSPACE; 5, 6 and 7 need in % 64 == 0)
 *   variant 7  as 5, but every tile whole (5 runs the tiles of a last, sparsely filled round as halves)
 *   variant 8  the left-hand side of Eq. 6 as ONE matrix product: a workgroup rebuilds the fine-tuned weight
 *              W + alpha S of its tile on the way to the matrix cores (alpha rounded to binary16, the sum rounded
 *              once to binary16, as a per-tenant fp16 model would store it) and multiplies once, 256 x 256
 *              tiles.  Half the matrix-core work of variants 4 to 7; the result differs from theirs by that
 *              rounding of the weights (about 2e-4 of the largest output at in = 4096) and equals, up to
 *              summation order, bd_linear_naive on bd_materialize'd weights.  Same conditions as 5. */
bd_status bd_linear_multitenant_variant(const uint16_t* x_f16, const uint16_t* w_base_f16,
                                        const uint32_t* const* packed_by_tenant,
                                        const float* alpha_by_tenant,
                                        const int32_t* tenant_of_token,
                                        uint16_t* y_f16,
                                        int64_t T, int64_t out, int64_t in, int32_t n_tenants,
                                        void* workspace, size_t workspace_bytes, void* stream,
                                        int32_t variant);

/* ---- serving layout ---------------------------------------------------------------------
 * Sec. 4.3 of the paper serves every fine-tune from one shared base plus packed 1-bit deltas
 * that stay packed until they are on the chip.  For that stream the library keeps both in a
 * TILED layout whose bytes are already in matrix-core operand order, so that every load of the
 * decode kernel is one contiguous 512 B or 1 KiB run.  Re-laying a tensor is done once, offline,
 * like compression.  The layout (tiles of 16 rows x 256 reduction elements, ordered [row block][k tile]):
 *   base   Wt[rb][kt][v][l][e] fp16 = W[16 rb + l%16][256 kt + 32 v + 8 (l/16) + e]    v<8, l<64, e<8
 *   signs  St[rb][kt][l][v]    byte,  bit e = packed sign of the same element
 * Rows beyond out and elements beyond in are zero.  Sizes come from bd_tiled_*_bytes (0 for
 * shapes the tiled path rejects: in % 32 != 0, or a tiled base of 4 GiB or more). */
size_t bd_tiled_base_bytes(int64_t out, int64_t in);
size_t bd_tiled_signs_bytes(int64_t out, int64_t in);

/* w_f16 [out, in] fp16 row-major -> w_tiled (bd_tiled_base_bytes(out, in) bytes). */
bd_status bd_tile_base(const uint16_t* w_f16, int64_t out, int64_t in, uint16_t* w_tiled, void* stream);

/* packed [out, in/32] as written by bd_compress / bd_pack_signs -> signs_tiled
 * (bd_tiled_signs_bytes(out, in) bytes). */
bd_status bd_tile_signs(const uint32_t* packed, int64_t out, int64_t in, uint32_t* signs_tiled, void* stream);

/* The multi-tenant linear of Eq. 6 over the serving layout; same arithmetic and rounding as
 * bd_linear_multitenant.
 *   w_tiled          tiled base (bd_tile_base)
 *   tiled_by_tenant  HOST array of n_tenants DEVICE pointers to tiled deltas (bd_tile_signs); the
 *                    pointers travel in the kernel arguments, so no device-side pointer table is read.
 *                    Entries of tenants without a token in this call may be NULL.
 *   alpha_by_tenant  device array of n_tenants floats
 *   tenant_of_token  HOST [T]; x_f16 [T, in]; y_f16 [T, out], must not overlap x or w_tiled.
 * Tokens are grouped by tenant inside the call, over the whole batch; up to 32 tokens are one launch
 * (two 16-column tiles that share the base registers), more run as several launches of 32 consecutive
 * tokens of the grouped order (the base is then streamed once per launch, a delta once per launch that
 * holds one of its tenant's tokens).  Needs no workspace. */
bd_status bd_linear_multitenant_tiled(const uint16_t* x_f16, const uint16_t* w_tiled,
                                      const uint32_t* const* tiled_by_tenant,
                                      const float* alpha_by_tenant,
                                      const int32_t* tenant_of_token,
                                      uint16_t* y_f16,
                                      int64_t T, int64_t out, int64_t in, int32_t n_tenants,
                                      void* stream);

/* The prefill regime of Sec. 4.3 (many tokens per tenant) on the SAME serving layout, so that one copy of the base and
 * of every delta serves both decode and prefill: all T tokens (1 <= T <= 65535) in ONE matrix-core GEMM launch, tokens
 * sorted by tenant and cut into tiles that never mix tenants (as bd_linear_multitenant does with a workspace).
 *   one_product == 0  Eq. 6 as written: base product and +-1 product in separate binary32 accumulators, alpha applied to
 *                     the finished sum (128 x 256 tiles; the arithmetic of bd_linear_multitenant's GEMM)
 *   one_product != 0  its left-hand side, X (W + alpha S) with the bracket rounded once to binary16 (256 x 256 tiles;
 *                     the arithmetic of variant 8 of bd_linear_multitenant_variant): half the matrix-core work
 *   tiled_by_tenant   HOST array of n_tenants DEVICE pointers (bd_tile_signs); NULL allowed for tenants without a token
 *   workspace         bd_workspace_bytes(BD_OP_LINEAR_TILED_GEMM, T, out, in, n_tenants) bytes, 256-byte aligned, device
 *                     memory: receives the token tables and the pointer table of this call (one call at a time per workspace)
 * in % 64 == 0 (else BD_ERR_UNSUPPORTED); y must not overlap x or w_tiled.  A batch with few tokens per tenant is
 * cheaper through bd_linear_multitenant_tiled (a GEMM tile holds one tenant's tokens only).  Asynchronous. */
bd_status bd_linear_multitenant_tiled_gemm(const uint16_t* x_f16, const uint16_t* w_tiled,
                                           const uint32_t* const* tiled_by_tenant,
                                           const float* alpha_by_tenant,
                                           const int32_t* tenant_of_token,
                                           uint16_t* y_f16,
                                           int64_t T, int64_t out, int64_t in, int32_t n_tenants,
                                           int32_t one_product,
                                           void* workspace, size_t workspace_bytes, void* stream);

/* Up to 3 linears that read the same activations (q, k, v or gate, up of one decoder layer) in
 * ONE launch: y_m = Eq. 6 with matrix m's base, deltas and scales, for m < n_mats.
 *   w_tiled             HOST [n_mats] of device pointers
 *   tiled_by_mat_tenant HOST [n_mats * n_tenants], entry m * n_tenants + e = tenant e's delta of matrix m
 *   alpha_by_mat        HOST [n_mats] of device arrays [n_tenants]
 *   y_f16               HOST [n_mats] of device pointers, y_m is [T, out[m]]
 *   out                 HOST [n_mats]; `in`, x, T and tenant_of_token are shared. */
bd_status bd_linear_multitenant_tiled_group(int32_t n_mats, const uint16_t* x_f16,
                                            const uint16_t* const* w_tiled,
                                            const uint32_t* const* tiled_by_mat_tenant,
                                            const float* const* alpha_by_mat,
                                            const int32_t* tenant_of_token,
                                            uint16_t* const* y_f16,
                                            int64_t T, const int64_t* out, int64_t in, int32_t n_tenants,
                                            void* stream);

/* ---- several sign planes per tenant (Sec. 4.2 of the paper, ablation over the fidelity of Delta) ----
 * Applying the compressor again with the compressed model as the base gives a second 1-bit mask
 * with a scale of its own, and so on: W_fine ~ W_base + sum_{j<k} alpha_j S_j.  The residual
 *   r_0 = f32(w_ft) - f32(w_base),   r_{j+1} = r_j - alpha_j * Sign(r_j)          (IEEE binary32)
 * is never re-rounded to fp16; plane j = sign bits of r_j (Eq. 2), alpha_j = fp16_rne(mean |r_j|)
 * (Eq. 4, binary64 sum).  k = 1 is bd_compress.
 *   packed [k][out][in/32]; alpha: k floats on the device (also read back by later iterations);
 *   workspace as for bd_compress; 1 <= k <= BD_MAX_PLANES, else BD_ERR_SHAPE.  (Plane j starts
 *   j * out * in / 8 bytes into packed: 16-byte aligned, as bd_tile_signs wants it, when out*in % 128 == 0.)
 * Asynchronous: k compress launches, each reading the scales the earlier ones left in `alpha`. */
#define BD_MAX_PLANES 8
bd_status bd_compress_iterated(const uint16_t* w_base_f16, const uint16_t* w_ft_f16,
                               int64_t out, int64_t in, int32_t k,
                               uint32_t* packed, float* alpha,
                               void* workspace, size_t workspace_bytes, void* stream);

/* Eq. 6 with k planes per tenant on the row-major tensors (the k-plane form of bd_linear_multitenant):
 *   y[t] = x[t] W_base^T + sum_{j<k} alpha[e*k+j] * (x[t] S_{e,j}^T),   e = tenant_of_token[t]
 *   planes_by_tenant  DEVICE array [n_tenants * k] of device pointers, entry e*k + j = plane j of tenant e as
 *                     bd_compress_iterated writes it ([out, in/32] words)
 *   alpha_by_tenant   device [n_tenants * k]
 * Runs on the matrix-core decode kernel only: in % 128 == 0 and a base below 4 GiB, else BD_ERR_UNSUPPORTED.
 * A token occupies k of a launch's 32 columns; more tokens run as several launches.  Other arguments and errors as
 * bd_linear_multitenant; k outside 1..BD_MAX_PLANES gives BD_ERR_SHAPE.  Needs no workspace. */
bd_status bd_linear_multitenant_kbit(const uint16_t* x_f16, const uint16_t* w_base_f16,
                                     const uint32_t* const* planes_by_tenant,
                                     const float* alpha_by_tenant,
                                     const int32_t* tenant_of_token,
                                     uint16_t* y_f16,
                                     int64_t T, int64_t out, int64_t in, int32_t n_tenants, int32_t k,
                                     void* stream);

/* Eq. 6 over the 8-bit base (Sec. 4.2, quantized base models) on the row-major tensors, the decode form:
 *   y[t,n] = wscale[n] * sum_k x[t,k] q[n,k] + alpha[e] * (x[t] S_e^T)[n],   e = tenant_of_token[t]
 *   q [out, in] int8 and wscale [out] binary32 as bd_quantize_base_q8 writes them, packed_by_tenant / alpha_by_tenant as
 *   for bd_linear_multitenant (deltas from bd_compress_q8).  Runs on the matrix-core decode kernel: in % 128 == 0 and
 *   out * in < 2^32, else BD_ERR_UNSUPPORTED; 32 tokens per launch, more tokens run as several launches (many tokens
 *   per tenant: bd_linear_multitenant_gemm_q8).  Needs no workspace.  Other arguments and errors as
 *   bd_linear_multitenant. */
bd_status bd_linear_multitenant_q8(const uint16_t* x_f16, const int8_t* q, const float* wscale,
                                   const uint32_t* const* packed_by_tenant, const float* alpha_by_tenant,
                                   const int32_t* tenant_of_token, uint16_t* y_f16,
                                   int64_t T, int64_t out, int64_t in, int32_t n_tenants, void* stream);

/* The GEMM form (the prefill regime of Sec. 4.3, many tokens per tenant) of the two extensions of Sec. 4.2, for any
 * T >= 1 (T <= 65535): tokens are sorted by tenant and cut into tiles of 128 rows that never mix tenants, every tile
 * is a matrix-core GEMM over `in` (128 x 128 tiles of y).  Tensors row-major as bd_compress_iterated /
 * bd_quantize_base_q8 + bd_compress_q8 write them; in % 32 == 0.
 *   workspace   bd_workspace_bytes(BD_OP_LINEAR_GEMM, T, out, in, n_tenants) bytes, 256-byte aligned, device memory;
 *               holds the token tables of this call until the launch has run (one call at a time per workspace)
 * _gemm_kbit (fidelity of Delta, k planes): y[t] = x[t] W_base^T + x[t] D_e^T with D_e = sum_j alpha[e*k+j] S_{e,j}
 *   added up in fp16 in ascending j (one rounding per plane; 2^-11 of the delta term against the exact sum);
 *   planes_by_tenant, alpha_by_tenant as for bd_linear_multitenant_kbit; k outside 1..BD_MAX_PLANES: BD_ERR_SHAPE.
 * _gemm_q8 (quantized base models): y[t,n] = wscale[n] * sum_k x[t,k] q[n,k] + alpha[e] * (x[t] S_e^T)[n];
 *   q [out, in] int8, wscale [out] binary32 (device), packed_by_tenant / alpha_by_tenant as for bd_linear_multitenant.
 * Errors as bd_linear_multitenant, BD_ERR_WORKSPACE for a missing, small or misaligned workspace, BD_ERR_UNSUPPORTED
 * for in == 0.  Asynchronous. */
bd_status bd_linear_multitenant_gemm_kbit(const uint16_t* x_f16, const uint16_t* w_base_f16,
                                          const uint32_t* const* planes_by_tenant, const float* alpha_by_tenant,
                                          const int32_t* tenant_of_token, uint16_t* y_f16,
                                          int64_t T, int64_t out, int64_t in, int32_t n_tenants, int32_t k,
                                          void* workspace, size_t workspace_bytes, void* stream);
bd_status bd_linear_multitenant_gemm_q8(const uint16_t* x_f16, const int8_t* q, const float* wscale,
                                        const uint32_t* const* packed_by_tenant, const float* alpha_by_tenant,
                                        const int32_t* tenant_of_token, uint16_t* y_f16,
                                        int64_t T, int64_t out, int64_t in, int32_t n_tenants,
                                        void* workspace, size_t workspace_bytes, void* stream);

/* Eq. 6 with k planes per tenant over the serving layout:
 *   y[t] = x[t] W_base^T + sum_{j<k} alpha[e*k+j] * (x[t] S_{e,j}^T),   e = tenant_of_token[t]
 * (each +-1 sum accumulated in binary32, scaled, added to the base product; one rounding to fp16).
 *   planes_by_tenant  HOST [n_tenants * k] of DEVICE pointers, entry e*k + j = tiled plane j of tenant e
 *                     (bd_tile_signs of packed plane j); NULL allowed for tenants without a token
 *   alpha_by_tenant   device [n_tenants * k]
 * A token occupies k of a launch's 32 columns, so one launch covers 2 * floor(16 / k) tokens; more
 * tokens run as several launches.  k = 1 is bd_linear_multitenant_tiled.  Other arguments and errors
 * as there; k outside 1..BD_MAX_PLANES gives BD_ERR_SHAPE. */
bd_status bd_linear_multitenant_tiled_kbit(const uint16_t* x_f16, const uint16_t* w_tiled,
                                           const uint32_t* const* planes_by_tenant,
                                           const float* alpha_by_tenant,
                                           const int32_t* tenant_of_token,
                                           uint16_t* y_f16,
                                           int64_t T, int64_t out, int64_t in, int32_t n_tenants, int32_t k,
                                           void* stream);

/* The grouped launch with k planes per tenant: planes_by_mat_tenant HOST [n_mats * n_tenants * k],
 * entry (m * n_tenants + e) * k + j; alpha_by_mat HOST [n_mats] of device arrays [n_tenants * k]. */
bd_status bd_linear_multitenant_tiled_group_kbit(int32_t n_mats, const uint16_t* x_f16,
                                                 const uint16_t* const* w_tiled,
                                                 const uint32_t* const* planes_by_mat_tenant,
                                                 const float* const* alpha_by_mat,
                                                 const int32_t* tenant_of_token,
                                                 uint16_t* const* y_f16,
                                                 int64_t T, const int64_t* out, int64_t in, int32_t n_tenants,
                                                 int32_t k, void* stream);

/* ---- 8-bit base (Sec. 4.2 of the paper, "Quantized base models") ---------------------------------
 * Only the base weights are quantised: activations, fine-tuned weights, deltas and scales stay as they
 * are.  The quantiser is 8-bit round-to-nearest with one scale per output row:
 *   scale[n] = max_k |W[n,k]| / 127 (binary32; 1 for an all-zero row)
 *   q[n,k]   = clamp(round_to_nearest_even(W[n,k] / scale[n]), -127, 127)
 * and the base that deltas are taken against and that Eq. 6 multiplies is scale[n] * q[n,k] in
 * binary32.  The base stream of the decode kernel halves, so at 16 tenants the deltas are two thirds
 * of the bytes.
 *   q [out, in] int8 row-major, scale [out] float, both on the device. */
bd_status bd_quantize_base_q8(const uint16_t* w_f16, int64_t out, int64_t in, int8_t* q, float* scale, void* stream);

/* The compressor of Sec. 3.1 against the quantised base: Delta = f32(w_ft) - scale[n] * q[n,k].
 * Arguments, workspace and errors as bd_compress (q must be 8-byte aligned). */
bd_status bd_compress_q8(const int8_t* q, const float* scale, const uint16_t* w_ft_f16, int64_t out, int64_t in,
                         uint32_t* packed, float* alpha, void* workspace, size_t workspace_bytes, void* stream);

/* Serving layout of the 8-bit base: tiles of 16 rows x 256 k, one byte u = q + 128 per weight,
 *   Wq[rb][kt][i][l][h][e] = 128 + q[16 rb + l%16][256 kt + 32 (2 i + h) + 8 (l/16) + e]   i<4, l<64, h<2, e<8
 * followed by the scales, 16 floats per row block (zeros beyond out).  bd_tiled_base_q8_bytes gives the
 * size of the whole tensor (0 for shapes the tiled path rejects). */
size_t bd_tiled_base_q8_bytes(int64_t out, int64_t in);
bd_status bd_tile_base_q8(const int8_t* q, const float* scale, int64_t out, int64_t in, void* wq_tiled, void* stream);

/* bd_linear_multitenant_tiled / _group over an 8-bit base (wq_tiled from bd_tile_base_q8; the deltas must
 * have been compressed against the same quantised base, bd_compress_q8).  Same arguments otherwise. */
bd_status bd_linear_multitenant_tiled_q8(const uint16_t* x_f16, const void* wq_tiled,
                                         const uint32_t* const* tiled_by_tenant,
                                         const float* alpha_by_tenant,
                                         const int32_t* tenant_of_token,
                                         uint16_t* y_f16,
                                         int64_t T, int64_t out, int64_t in, int32_t n_tenants,
                                         void* stream);
bd_status bd_linear_multitenant_tiled_group_q8(int32_t n_mats, const uint16_t* x_f16,
                                               const void* const* wq_tiled,
                                               const uint32_t* const* tiled_by_mat_tenant,
                                               const float* const* alpha_by_mat,
                                               const int32_t* tenant_of_token,
                                               uint16_t* const* y_f16,
                                               int64_t T, const int64_t* out, int64_t in, int32_t n_tenants,
                                               void* stream);

/* ---- delta images: storing a tenant's delta and swapping it in while serving ----------------
 * Sec. 3.3 of the paper: a 1-bit delta is small enough to be kept per tenant on disk or in host
 * memory and loaded on demand.  A delta IMAGE holds one tenant's whole compressed model (every
 * matrix's k sign planes, row-major packed as bd_compress(_iterated) writes them, and scales) as one
 * relocatable block of bytes: the file format and, unchanged, the pinned staging buffer of a swap.
 * Layout (little-endian):
 *   0  char[8] "BDLTv001" | 8 u32 n_mats | 12 u32 planes k | 16 u64 total bytes
 *   24 u64 sum of the payload's 64-bit words | 32 entry[n_mats] { i64 out, in; u64 packed_offset,
 *   packed_bytes, alpha_offset } | f32 alpha[n_mats][k] | pad to 256 | per matrix, 256-byte aligned:
 *   u32 packed[k][out][in/32].
 * All image and file calls run on the HOST and take host pointers.  A swap is then
 *   bd_delta_file_read (or any other way of getting the bytes into pinned host memory)
 *   bd_delta_upload     one asynchronous host-to-device copy of the whole image into an arena
 *   bd_delta_install    re-tiles every plane from the arena into the serving layout and writes the
 *                       tenant's scales into the per-matrix scale arrays, on the same stream;
 * the linears may use the new pointers once that stream has reached this point (an event of the
 * caller's).  Decode keeps running on another stream meanwhile; nothing here synchronises. */
#define BD_DELTA_MAX_MATS 4096

/* Bytes of the image for these matrices (0 for invalid arguments). out, in: HOST [n_mats]. */
size_t bd_delta_image_bytes(int32_t n_mats, const int64_t* out, const int64_t* in, int32_t k);

/* Writes the image into `image` (exactly bd_delta_image_bytes long, else BD_ERR_WORKSPACE).
 * packed: HOST [n_mats] of HOST pointers to [k][out][in/32] words; alpha: HOST [n_mats] of HOST [k]. */
bd_status bd_delta_image_build(void* image, size_t image_bytes, int32_t n_mats, const int64_t* out,
                               const int64_t* in, int32_t k, const uint32_t* const* packed,
                               const float* const* alpha);

/* Validates header and entry table against `bytes` (and the checksum if asked); returns n_mats, k. */
bd_status bd_delta_image_check(const void* image, size_t bytes, int32_t verify_checksum, int32_t* n_mats, int32_t* k);

/* Shape and offsets (from the start of the image) of matrix m; any output pointer may be NULL. */
bd_status bd_delta_image_entry(const void* image, size_t bytes, int32_t m, int64_t* out, int64_t* in,
                               size_t* packed_offset, size_t* alpha_offset);

/* File I/O: the file is the image, byte for byte.  bd_delta_file_bytes reads the size from the header. */
bd_status bd_delta_file_write(const char* path, const void* image, size_t bytes);
bd_status bd_delta_file_bytes(const char* path, size_t* bytes);
bd_status bd_delta_file_read(const char* path, void* image, size_t bytes);

/* image: HOST (pinned memory makes the copy truly asynchronous); arena: DEVICE, `bytes` long, 256-byte
 * aligned.  Enqueues one copy on `stream`. */
bd_status bd_delta_upload(const void* image, size_t bytes, void* arena, void* stream);

/* After bd_delta_upload on the same stream.  tiled_dst: HOST [n_mats * k] of DEVICE buffers of
 * bd_tiled_signs_bytes(out_m, in_m) bytes (entry m*k + j = plane j of matrix m); alpha_by_tenant:
 * HOST [n_mats] of DEVICE arrays [n_tenants * k], of which entries tenant*k .. tenant*k + k-1 are
 * written.  `image` must stay valid until the stream has passed this point. */
bd_status bd_delta_install(const void* image, size_t bytes, const void* arena, int32_t tenant, int32_t n_tenants,
                           uint32_t* const* tiled_dst, float* const* alpha_by_tenant, void* stream);

/* The grouping step of the linear, exposed so that a scheduler (or a test) can see it: the
 * tokens of one decode launch (T <= 32, all HOST arrays) sorted by tenant, stable, and cut
 * into jobs.  A job is one tenant's run of columns inside one 16-column tile; the kernel
 * streams a tenant's delta once per job, i.e. once per step unless a tenant's tokens straddle
 * the tile boundary.
 *   token_of_col[T]   column -> index into tenant_of_token
 *   job_tenant, job_tile, job_col_begin, job_col_end: [T] each, first *n_jobs entries valid;
 *   columns job_tile*16 + [job_col_begin, job_col_end) belong to the job.
 * T outside 1..32 gives BD_ERR_SHAPE. */
bd_status bd_group_tokens(const int32_t* tenant_of_token, int32_t T,
                          int32_t* token_of_col, int32_t* job_tenant, int32_t* job_tile,
                          int32_t* job_col_begin, int32_t* job_col_end, int32_t* n_jobs);

/* ---- measurement helpers (the naive system of Sec. 4.3 and bandwidth probes) ------------- */

/* w_out = fp16( f32(w_base) + alpha * s ), the full per-tenant matrix that the naive baseline
 * of Sec. 4.3 keeps for every fine-tune.  alpha: one float on the device. */
bd_status bd_materialize(const uint16_t* w_base_f16, const uint32_t* packed, const float* alpha,
                         uint16_t* w_out_f16, int64_t out, int64_t in, void* stream);

/* The naive forward pass of Sec. 4.3: token t is multiplied by its own tenant's full fp16
 * matrix.  w_by_tenant: device array of n_tenants device pointers, each [out, in] fp16.
 * tenant_of_token: HOST [T].  y_f16: [T, out]. */
bd_status bd_linear_naive(const uint16_t* x_f16, const uint16_t* const* w_by_tenant,
                          const int32_t* tenant_of_token, uint16_t* y_f16,
                          int64_t T, int64_t out, int64_t in, int32_t n_tenants, void* stream);

/* Streams `bytes` (a multiple of 16) from src with 128-bit loads and folds them into
 * sink[0..3] (4 x uint32 on the device) so the loads cannot be elided: the read ceiling every
 * bandwidth figure is also quoted against. */
bd_status bd_probe_read(const void* src, size_t bytes, uint32_t* sink, void* stream);

/* dst <- src, `bytes` a multiple of 16: a plain copy of known size, used to calibrate the
 * profiler's HBM byte counters. */
bd_status bd_probe_copy(void* dst, const void* src, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* BITDELTA_H */
