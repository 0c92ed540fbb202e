/*
 * w2mm -- 2-bit-weight mixed-precision matmul for AMD MI355X (gfx950 / CDNA4)
 *
 *     Y[M,N] = X[M,K] . dequant(W2[K,N])
 *
 * W2 holds 2-bit weight codes with one bf16 scale per group of G consecutive K
 * per output column.  X is either int8 (quantised per token by
 * w2_quantize_rows; "w2a8") or bf16 ("w2a16").  Y is bf16.
 *
 * Naming: X = activations (M tokens), W = weights (N output features).  The
 * paper names the weight matrix A (its M x K), the activations B (its N x K)
 * and the output C.
 *
 * Conventions for every entry point
 *   - returns a w2_status_t (0 = OK, negative = error); never throws, never
 *     aborts, never synchronises the device;
 *   - all work is enqueued on `stream` (a hipStream_t passed as void*, NULL =
 *     the default stream) of the CURRENT device;
 *   - every buffer is owned by the caller; the library keeps no device state
 *     (w2_matmul_a8_fused_noalloc, with its built-in scratch buffer, is the one
 *     exception), allocates nothing and holds no handles, so calls from several
 *     host threads are independent; which kernel runs depends on the arguments
 *     alone (the process environment is never read);
 *   - "dev" pointers are device memory of the current device, "host" pointers
 *     are ordinary host memory;
 *   - arguments are validated before anything is launched: a call that returns
 *     an error has written nothing;
 *   - M == 0 is valid everywhere and does nothing.
 *
 * Shape rules: K > 0, K % 256 == 0, G in {64, 128}; N > 0 and N % 8 == 0
 * (columns are padded to a multiple of 16 inside the packed blob);
 * `packed`, `xq`, `X` and `Y` 16-byte aligned, row strides (ldx, ldy) in
 * elements and multiples of 8.
 */
#ifndef W2MM_H
#define W2MM_H

#include <stddef.h>
#include <stdint.h>

#if defined(__GNUC__)
#define W2_API __attribute__((visibility("default")))
#else
#define W2_API
#endif

#ifdef __cplusplus
extern "C" {
#endif

/* Code -> value map of the canonical (caller-side) weight codes.  The paper
 * does not print one; these follow the benchmark configuration:
 * INT2: q = c - 2 (values -2,-1,0,1); TERNARY: q = c - 1 (values -1,0,1),
 * code 3 is illegal. */
typedef enum { W2_CODEC_INT2 = 0, W2_CODEC_TERNARY = 1 } w2_codec_t;

typedef enum { W2_DT_F32 = 0, W2_DT_BF16 = 1 } w2_dtype_t;

typedef enum {
    W2_OK = 0,
    W2_ERR_INVALID_ARG = -1,       /* NULL pointer, unknown enum, negative size */
    W2_ERR_UNSUPPORTED_SHAPE = -2, /* violates the shape rules above */
    W2_ERR_MISALIGNED = -3,        /* pointer or stride alignment */
    W2_ERR_BUFFER_TOO_SMALL = -4,  /* packed_bytes / workspace_bytes too small */
    W2_ERR_HIP = -5,               /* a HIP call failed; see w2_last_error() */
    W2_ERR_BAD_CODE = -6           /* reserved for callers that check bad_codes */
} w2_status_t;

/* Kernel families, for w2_matmul_a8_ex / w2_matmul_a16_ex and the debug export.
 * AUTO picks by shape.  w2a8: GEMV up to M = 8 wherever the rows fit a workgroup's local memory (up to 16
 * while two workgroups share a CU or the projection is narrow: N <= 10240 or at most 256 workgroups; up to 32
 * for K <= 4096), MIDM above it up to
 * M = 64 (128 when N <= 4096; 32 when N >= 24576 or, with a workspace, K >= 14336), else TILED (64-row
 * tiles; 128-row tiles from M = 1024, or from M = 128 where they fill the chip).
 * w2a16: GEMV up to M = 8 (up to 16 for K <= 4096; up to 4 for K > 5120 with N >= 32768) wherever the bf16
 * rows fit a workgroup's local memory, SMALLM for the rest up to M = 8 (M = 2 for K > 16384; M = 4 for
 * K > 8192 with a workspace), MIDM up to M = 64 (M = 128 when N <= 4096, M = 40 when N >= 32768), else the
 * SCALED16 tiled kernel.
 * GEMV: the decode kernel: whole rows in local memory, a wave streams a contiguous run of a column
 * block's tiles through a rolling register window into int8 MFMA (w2a8, M <= 32) or, with bf16 rows left as they
 * are and the zero-point weight construction, into bf16 MFMA (w2a16, M <= 16; W2_ERR_UNSUPPORTED_SHAPE when the
 * rows do not fit).
 * DOT4: per-lane v_dot4_i32_i8
 * with split-K across the waves of a workgroup (M <= 4; kept as the dot-product form of the microkernel,
 * selectable here).  SMALLM: one 16-row int8 (bf16 for a16) MFMA tile per
 * wave, split-K across waves (M <= 16).  MIDM: the weight stream
 * is still read once per band of 64 rows; every streamed tile is multiplied into one to four
 * 16-row MFMA tiles (M <= 256 = four bands; for w2a16 with the SCALED16 weight construction).
 * TILED: LDS-staged MFMA tiles (any M; for w2a16 the zero-point construction).
 * SCALED16 (w2a16 only): the weights are built as sw*q from code and group
 * scale (Sec. II-D, the alternative 16-bit construction) and go to the bf16
 * matrix instruction as they are: no zero-point term, no dequant step, one
 * fp32 accumulator per output over the whole K.  M <= 16: the SMALLM kernel
 * with this construction (never picked by AUTO: the zero-point form is faster
 * there); M <= 64: the MIDM kernel; above: a 128-row tiled kernel of its own,
 * AUTO's choice for prefill.  Needs bf16 scales with an exponent field below
 * 254 (-2 sw is made by raising the exponent by one). */
typedef enum { W2_VARIANT_AUTO = 0, W2_VARIANT_DOT4 = 1, W2_VARIANT_SMALLM = 2,
               W2_VARIANT_TILED = 3, W2_VARIANT_MIDM = 4, W2_VARIANT_SCALED16 = 5,
               W2_VARIANT_GEMV = 6 } w2_variant_t;

/* Overrides of the library's own choices, for tests and tuning sweeps; taken by
 * the *_ex / *_epi entry points, the debug export and the probe.  A NULL pointer,
 * or a field left 0, means the library's rule, which depends on the shape only.
 * A value a field does not allow gives W2_ERR_INVALID_ARG (nothing launched).
 * Fields that do not concern the kernel family that runs are ignored. */
typedef struct {
    int variant;          /* w2_variant_t: the kernel family */
    int dot4_max_m;       /* w2a8 AUTO: largest M given to DOT4 (1..4; default: never) */
    int midm_min_m;       /* AUTO: smallest / largest M given to MIDM (1..256) */
    int midm_max_m;
    int small_waves;      /* GEMV, DOT4, SMALLM: waves per workgroup, 1..16 */
    int small_cbw;        /* ... column blocks per workgroup: 1, 2, 4, 8 or 16, at most the waves */
    int small_kc;         /* ... k per local-memory chunk of the activations: a multiple of 256 */
    int gemv_window;      /* GEMV: weight tiles a wave keeps in flight: 2, 4 or 8 */
    int gemv_max_m;       /* w2a8 AUTO: largest M given to GEMV (1..32) */
    int midm_cbw;         /* MIDM: column blocks per workgroup: 2, 4 or 8 */
    int tiled_bm;         /* w2a8 TILED: rows per workgroup: 64 or 128 (128: G = 128) */
    int tiled_bn;         /* TILED / SCALED16 tiled kernels: columns per workgroup: 128 or 256 (w2a8, 64-row tiles: also 64) */
    int tiled_kw;         /* w2a8 TILED, 128-column workgroups: K ranges inside a workgroup: 1, 2 or 4 */
    int tiled_wd;         /* w2a8 TILED, 64-row tiles: weight stages in flight per wave: 2 or 8 */
    int tiled_group_m;    /* ... row tiles per band of the workgroup order: 1..1024 */
    int splitk;           /* tiled and mid-M kernels: 1 = never split K, n = 2..16: n parts if the workspace holds them */
    int splitk_min_tiles; /* ... planner: fewest 256-k tiles per part, 1..1024 */
    int stream_unroll;    /* w2_debug_stream_read: 1 KiB chunks in flight per wave: 4, 8 or 16 */
    int stream_blocks;    /* ... most workgroups launched: 1..65536 */
    int gemv_cbw;         /* GEMV: column blocks per workgroup, any number 1..16 (even for the gated epilogue) */
    int gemv_ks;          /* ... x K ranges per workgroup, 1..16: at most 16 waves (8 from five rows on, and for w2a16) */
    int fused_rows;       /* w2_matmul_a8_fused*: largest M quantised inside the matmul kernel, one launch (1..8) */
} w2_tuning_t;

/* ------------------------------------------------------------------------
 * Offline weight pre-formatting (Sec. II-B and II-D: the 2-bit weights are
 * packed into the instruction's layout once, before inference, at no run-time
 * cost).  The device layout
 * is this library's own (the paper's VNNI4-interleaved and VNNI16 layouts are
 * for x86 and Xe2); the principle kept from Sec. II-B is that one shift and
 * one mask land four consecutive-K codes directly in the byte lanes the int8
 * dot/matrix instruction consumes.
 * ------------------------------------------------------------------------ */

/* Size in bytes of the packed blob for a K x N weight with group size G.
 * bytes: host out-pointer. */
W2_API int w2_packed_size(int64_t K, int64_t N, int G, size_t* bytes);

/* codes_KN  dev, uint8, one code per byte, row-major [K][N]
 * scales    dev, bf16 bit patterns, row-major [K/G][N]
 * packed    dev, caller-allocated, >= w2_packed_size bytes, 16-byte aligned;
 *           fully overwritten (padding columns get value 0 and scale 0)
 * bad_codes dev, int32 counter or NULL; if given it must be zero on entry and
 *           is incremented once per code outside the codec's alphabet
 *           (> 3, or == 3 under TERNARY).  Such a code is stored as value 0. */
W2_API int w2_prepack(const uint8_t* codes_KN, const uint16_t* scales, int64_t K, int64_t N, int G,
               w2_codec_t codec, void* packed, size_t packed_bytes, int32_t* bad_codes,
               void* stream);

/* ------------------------------------------------------------------------
 * Per-token activation quantisation (Sec. II-B; Sec. II-D: abs-max per
 * granularity gives the scale, entries are multiplied by the inverse scale
 * and converted to int8).  Granularity: one scale per row over all K.
 * All arithmetic in IEEE binary32, one rounding per operation:
 *   amax = max_k |x|;  inv = 127/amax;  sx = amax/127  (both 0 if amax == 0)
 *   xq = clamp(round_half_even(x * inv), -127, 127)
 * X     dev, [M][K] row-major with row stride ldx, fp32 or bf16 (x_dtype)
 * xq    dev, int8 [M][K] dense
 * sx    dev, fp32 [M]
 * gsum  dev, int32 [M][K/G] = per-group sums of xq, or NULL (then G is unused).
 *       The matmul calls do not need it; it is offered to callers that fold a
 *       weight zero-point themselves. */
W2_API int w2_quantize_rows(const void* X, w2_dtype_t x_dtype, int64_t M, int64_t K, int64_t ldx, int G,
                     int8_t* xq, float* sx, int32_t* gsum, void* stream);

/* ------------------------------------------------------------------------
 * w2a8 (Sec. II-C "up-convert and compute": 2-bit codes -> int8 in registers,
 * int8 x int8 -> int32; Sec. II-D: int32 -> float, x (activation scale x
 * weight scale), -> bf16, fused before the store):
 *   acc[m,g,n] = sum_{k in group g} xq[m,k] * q[k,n]            (int32, exact)
 *   Y[m,n]     = bf16( sx[m] * sum_g sw[g,n] * float(acc[m,g,n]) )   (fp32)
 * packed  dev, from w2_prepack with the same K, N, G
 *         Weight scales: finite bf16 with |sw| < 2^63 (for M > 8 the kernels
 *         multiply by sw * 2^64 in fp32); results below the fp32 normal range
 *         (|sx * sw * acc| < 2^-126) may lose precision.
 * xq, sx  dev, as produced by w2_quantize_rows ([M][K] dense, [M])
 * Y       dev, bf16 bit patterns [M][N], row stride ldy
 * workspace  optional (NULL / 0: none), dev, 16-byte aligned, contents
 *            undefined before and after: on shapes with few output tiles
 *            and a deep K (M > 32: the tiled kernel; 4 <= M <= 128 and
 *            K >= 13568: the mid-M kernel) K is split across workgroups
 *            (Sec. II-D, K-splitting for the smaller GEMM shapes) if there
 *            is room for the fp32 partial results (w2_workspace_size; less
 *            room = fewer parts or none, same result contract).  A second
 *            launch on `stream` sums the parts in a fixed order.  Not
 *            touched otherwise. */
W2_API int w2_matmul_a8(const void* packed, int64_t K, int64_t N, int G, const int8_t* xq,
                 const float* sx, int64_t M, uint16_t* Y, int64_t ldy, void* workspace,
                 size_t workspace_bytes, void* stream);

/* Same, with overrides (tests, tuning; tune == NULL: exactly w2_matmul_a8).  Returns
 * W2_ERR_UNSUPPORTED_SHAPE if a forced kernel family does not cover M. */
W2_API int w2_matmul_a8_ex(const void* packed, int64_t K, int64_t N, int G, const int8_t* xq,
                    const float* sx, int64_t M, uint16_t* Y, int64_t ldy, void* workspace,
                    size_t workspace_bytes, const w2_tuning_t* tune, void* stream);

/* The int2 x {fp32, bf16} -> bf16 call (Sec. II-D: activation quantisation
 * fused into the GEMM; Sec. III-C: fusing wins for matrix-vector shapes, a
 * separate abs-max pass for multi-row activations).  Takes the unquantised
 * activations (fp32 or bf16, row stride ldx) and produces what
 * w2_quantize_rows followed by w2_matmul_a8 produces: the same int8 rows and
 * scales, and the same bf16 result bit for bit wherever the two calls cut K
 * into the same ranges (the fp32 partial sums of a column are then added in
 * the same order); where they do not (another workgroup shape for the same
 * M, or K split across workgroups, see w2_matmul_a8's workspace) the two
 * agree to the tolerance of the result contract.
 *   M <= 4 (M <= 8 when K <= 4096): one launch where a workgroup can hold the
 *           rows (M', M rounded up to a power of two: M'*K*elem_size up to
 *           128 KiB in registers and M*K up to about 150 KB of int8 rows in
 *           local memory): the abs-max is reduced per workgroup, redundantly,
 *           and the rows are quantised into local memory.  (M > 4 still asks
 *           for the workspace below, used or not.)
 *   Otherwise, with a workspace of w2_workspace_size(M, K, N, G, 0) bytes (dev,
 *           16-byte aligned; holds the int8 rows and their scales, contents
 *           undefined afterwards) two launches: quantise, then the kernel family
 *           w2_matmul_a8 picks for M.  Without one: W2_ERR_UNSUPPORTED_SHAPE,
 *           nothing launched; with one that is too small for M > 4:
 *           W2_ERR_BUFFER_TOO_SMALL. */
W2_API int w2_matmul_a8_fused(const void* packed, int64_t K, int64_t N, int G, const void* X,
                              w2_dtype_t x_dtype, int64_t ldx, int64_t M, uint16_t* Y, int64_t ldy,
                              void* workspace, size_t workspace_bytes, void* stream);

/* For callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid it): w2_matmul_a8_fused with the
 * workspace replaced by a buffer built into the library, W2_NOALLOC_SCRATCH_MIB
 * MiB of device memory per GPU that exists from the moment the library is loaded
 * on that GPU until the process ends.  The call itself allocates nothing, on the
 * device or on the host.  Same arguments, same results as w2_matmul_a8_fused
 * called with a workspace of that size (bit for bit).
 *   - The int8 rows and their scales must fit: M*K + 4*M (rounded up to 256)
 *     <= W2_NOALLOC_SCRATCH_MIB MiB, else W2_ERR_BUFFER_TOO_SMALL and nothing is
 *     launched.  What remains is offered to the tiled kernel for split-K.
 *   - Every call on a GPU shares that GPU's buffer: calls that may overlap on one
 *     GPU (different streams, different host threads) race; calls on one stream,
 *     or ordered by events, do not.  The buffer keeps the last call's contents;
 *     nothing in it needs clearing, every byte read was written by the same call.
 *   - The buffer's address is looked up once per GPU, by the first call there or
 *     by w2_init() (call it, with the device current, before a graph capture that
 *     contains the first call). */
#define W2_NOALLOC_SCRATCH_MIB 24
W2_API int w2_init(void);
W2_API int w2_matmul_a8_fused_noalloc(const void* packed, int64_t K, int64_t N, int G, const void* X,
                                      w2_dtype_t x_dtype, int64_t ldx, int64_t M, uint16_t* Y, int64_t ldy,
                                      void* stream);

/* Fused epilogues (Sec. II-D: further operations such as a bias addition or a
 * post-GEMM activation function are applied while the outputs are still in
 * registers, before the store).  With z[m,n] the fp32 result of the call
 * before rounding, plus bias[n] when bias is not NULL (dev, bf16 bit patterns
 * [N]):
 *   W2_ACT_NONE      Y[m,n] = bf16(z[m,n])
 *   W2_ACT_SILU      Y[m,n] = bf16(z * sigmoid(z))
 *   W2_ACT_SILU_MUL  the gated MLP form: the matrix holds gate and up
 *                    projections interleaved in blocks of 16 columns (block 2b =
 *                    gate columns 16b..16b+15, block 2b+1 = the up columns of the
 *                    same indices; the caller orders the columns so before
 *                    w2_prepack), N % 32 == 0, and Y has N/2 columns:
 *                    Y[m,16b+l] = bf16( silu(z[m,32b+l]) * z[m,32b+16+l] ),
 *                    ldy >= N/2.
 * epi == NULL is W2_ACT_NONE without bias.  Everything else as w2_matmul_a8_ex,
 * w2_matmul_a8_fused and w2_matmul_a16_ex (declared below). */
typedef enum { W2_ACT_NONE = 0, W2_ACT_SILU = 1, W2_ACT_SILU_MUL = 2 } w2_act_t;
typedef struct {
    const uint16_t* bias;
    int act;                /* w2_act_t */
} w2_epilogue_t;
W2_API int w2_matmul_a8_epi(const void* packed, int64_t K, int64_t N, int G, const int8_t* xq,
                            const float* sx, int64_t M, uint16_t* Y, int64_t ldy,
                            const w2_epilogue_t* epi, void* workspace, size_t workspace_bytes,
                            const w2_tuning_t* tune, void* stream);
W2_API int w2_matmul_a8_fused_epi(const void* packed, int64_t K, int64_t N, int G, const void* X,
                                  w2_dtype_t x_dtype, int64_t ldx, int64_t M, uint16_t* Y, int64_t ldy,
                                  const w2_epilogue_t* epi, void* workspace, size_t workspace_bytes,
                                  const w2_tuning_t* tune, void* stream);

/* ------------------------------------------------------------------------
 * w2a16 (Sec. II-D, "Alternative implementation": weights rebuilt as 16-bit
 * values from code and group scale, activations left unquantised, 16-bit
 * matrix instructions with fp32 accumulation, no quantise/dequantise):
 *   Y[m,n] = bf16( sum_k x[m,k] * (sw[k/G,n] * q[k,n]) )
 * X  dev, bf16 bit patterns [M][K], row stride ldx.
 * workspace  optional, as for w2_matmul_a8 (w2_workspace_size with a16 = 1). */
W2_API int w2_matmul_a16(const void* packed, int64_t K, int64_t N, int G, const uint16_t* X,
                  int64_t ldx, int64_t M, uint16_t* Y, int64_t ldy, void* workspace,
                  size_t workspace_bytes, void* stream);

W2_API int w2_matmul_a16_ex(const void* packed, int64_t K, int64_t N, int G, const uint16_t* X,
                     int64_t ldx, int64_t M, uint16_t* Y, int64_t ldy, void* workspace,
                     size_t workspace_bytes, const w2_tuning_t* tune, void* stream);

/* w2_matmul_a16_ex with a fused epilogue (see w2_epilogue_t above). */
W2_API int w2_matmul_a16_epi(const void* packed, int64_t K, int64_t N, int G, const uint16_t* X,
                             int64_t ldx, int64_t M, uint16_t* Y, int64_t ldy,
                             const w2_epilogue_t* epi, void* workspace, size_t workspace_bytes,
                             const w2_tuning_t* tune, void* stream);

/* Bytes of workspace (host out-pointer) with which the calls take their fastest
 * route for this problem.  a16 = 0 (w2_matmul_a8_fused; w2_matmul_a8 uses the
 * split-K part only and accepts the same buffer): room for the int8 rows and
 * their scales, rounded up to 256 bytes (0 where one launch covers the
 * quantisation: one or two rows of up to 64 KiB as fp32), plus, where a
 * kernel would split K, 2..16 fp32 copies of the M x N output.  a16 = 1
 * (w2_matmul_a16): the split-K part alone.  0 means no workspace is used. */
W2_API int w2_workspace_size(int64_t M, int64_t K, int64_t N, int G, int a16, size_t* bytes);

/* ------------------------------------------------------------------------
 * Test-only exports.
 * w2_debug_group_acc_a8: the int32 group accumulators acc[M][K/G][N] (dense)
 *   exactly as the chosen kernel family holds them before the dequant step.
 * w2_debug_unpack: inverse of w2_prepack: canonical codes [K][N] and scales
 *   [K/G][N] recovered from the blob (codec selects the code -> value map). */
W2_API int w2_debug_group_acc_a8(const void* packed, int64_t K, int64_t N, int G, const int8_t* xq,
                          int64_t M, const w2_tuning_t* tune, int32_t* acc, void* stream);
W2_API int w2_debug_unpack(const void* packed, int64_t K, int64_t N, int G, w2_codec_t codec,
                    uint8_t* codes_KN, uint16_t* scales, void* stream);

/* Streaming-read probe: 128-bit loads over `bytes` of dev memory, xor-reduced
 * into sink[0] (dev, uint32).  Used by the benchmark as the attainable
 * read-bandwidth ceiling the weight stream is compared with (the role the
 * int8-weight GEMV plays in Sec. III-B/III-C). */
W2_API int w2_debug_stream_read(const void* src, size_t bytes, uint32_t* sink, const w2_tuning_t* tune,
                                void* stream);

/* Comparator for the benchmark, not part of the method: an int8-weight GEMV
 * (Sec. III-B, III-C read the 2-bit GEMV against the int8 one, which moves
 * four times the bytes and has no up-convert).  W8: dev int8 [N][K] row-major
 * (16-byte aligned, K % 16 == 0, K <= 49152); xq: dev int8 [K] (16-byte
 * aligned); out: dev int32 [N], out[n] = sum_k W8[n][k] * xq[k], exact.
 * Launches on `stream`; writes nothing on error. */
W2_API int w2_debug_int8_gemv(const int8_t* W8, int64_t K, int64_t N, const int8_t* xq, int32_t* out,
                              void* stream);

W2_API const char* w2_status_string(int status);
/* Thread-local detail of the last error on this host thread (e.g. the HIP error
 * string or the violated rule); empty string if none. */
W2_API const char* w2_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* W2MM_H */
