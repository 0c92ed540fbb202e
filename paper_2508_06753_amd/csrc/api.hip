// C-ABI entry points of libw2mm: argument validation, dispatch by M, error
// reporting.  No arithmetic of the method lives here.
#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>

#include "../../include/w2mm.h"
#include "w2_internal.h"

namespace w2 {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
}

int check_launch(const char* what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error("%s: %s", what, hipGetErrorString(e));
        return W2_ERR_HIP;
    }
    return W2_OK;
}

namespace {
struct LdsGrant { const void* kern; int dev; size_t bytes; };
std::mutex g_lds_mutex;
constexpr int MAX_LDS_GRANTS = 512;         // fixed table: the bookkeeping never allocates
LdsGrant g_lds_grants[MAX_LDS_GRANTS];
int g_n_lds_grants = 0;
}  // namespace

int ensure_dynamic_lds(const void* kern, size_t bytes, const char* what)
{
    if (bytes <= 64 * 1024) return W2_OK;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) dev = 0;
    std::lock_guard<std::mutex> lock(g_lds_mutex);
    LdsGrant* g = nullptr;
    for (int i = 0; i < g_n_lds_grants; ++i)
        if (g_lds_grants[i].kern == kern && g_lds_grants[i].dev == dev) { g = &g_lds_grants[i]; break; }
    if (g && g->bytes >= bytes) return W2_OK;
    const hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) {
        set_error("%s: hipFuncSetAttribute(%zu bytes of LDS): %s", what, bytes, hipGetErrorString(e));
        return W2_ERR_HIP;
    }
    if (g) g->bytes = bytes;
    else if (g_n_lds_grants < MAX_LDS_GRANTS) g_lds_grants[g_n_lds_grants++] = {kern, dev, bytes};
    return W2_OK;                                            // a full table only means the call is repeated next time
}

// Streaming-read probe.  Each wave reads U consecutive 1 KiB chunks (one
// 128-bit load per lane per chunk) with all U loads in flight before any is
// consumed, then strides on; the loaded words are xor-reduced.
template <int U>
__global__ void __launch_bounds__(256)
stream_read_kernel(const uint4* __restrict__ src, size_t n_chunks, uint32_t* __restrict__ sink)
{
    uint32_t x = 0;
    const int lane = threadIdx.x & 63;
    const size_t gwave = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const size_t n_waves = ((size_t)gridDim.x * blockDim.x) >> 6;
    for (size_t base = gwave * U; base < n_chunks; base += n_waves * U) {
        uint4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t c = base + u < n_chunks ? base + u : n_chunks - 1;
            typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // non-temporal, as the GEMV kernels load their weights
            const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src + c * 64 + lane));
            v[u] = make_uint4(t[0], t[1], t[2], t[3]);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) x ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x ^= __shfl_xor(x, off);
    if (lane == 0 && x == 0x9e3779b9u) atomicXor(sink, x);   // keeps the loads alive; rarely taken
}

int launch_stream_read(const void* src, size_t bytes, uint32_t* sink, const w2_tuning_t& tune, hipStream_t stream)
{
    const size_t n_chunks = bytes / 1024;
    if (n_chunks == 0) return W2_OK;
    const int unroll = tune.stream_unroll ? tune.stream_unroll : 8;          // validated: 4, 8 or 16
    const size_t cap = tune.stream_blocks ? (size_t)tune.stream_blocks : 2048;
    size_t blocks = (n_chunks + 4 * (size_t)unroll - 1) / (4 * (size_t)unroll);   // 4 waves per block
    if (blocks > cap) blocks = cap;
    const dim3 grid((unsigned)blocks), block(256);
    if (unroll >= 16)
        hipLaunchKernelGGL(stream_read_kernel<16>, grid, block, 0, stream, (const uint4*)src, n_chunks, sink);
    else if (unroll >= 8)
        hipLaunchKernelGGL(stream_read_kernel<8>, grid, block, 0, stream, (const uint4*)src, n_chunks, sink);
    else
        hipLaunchKernelGGL(stream_read_kernel<4>, grid, block, 0, stream, (const uint4*)src, n_chunks, sink);
    return check_launch("w2_debug_stream_read");
}

static int fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

static bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

static int check_epilogue(const char* fn, const Epilogue& e, int64_t N)
{
    if (e.act < ACT_NONE || e.act > ACT_SILU_MUL) return fail(W2_ERR_INVALID_ARG, "%s: unknown activation %d", fn, e.act);
    if (e.act == ACT_SILU_MUL && N % 32)
        return fail(W2_ERR_UNSUPPORTED_SHAPE, "%s: the gated epilogue pairs 16-column blocks: N must be a multiple of 32", fn);
    return W2_OK;
}

static int check_shape(const char* fn, int64_t K, int64_t N, int G)
{
    if (K <= 0 || N <= 0) return fail(W2_ERR_INVALID_ARG, "%s: K and N must be positive", fn);
    if (G != 64 && G != 128) return fail(W2_ERR_UNSUPPORTED_SHAPE, "%s: G must be 64 or 128", fn);
    if (K % TILE_K) return fail(W2_ERR_UNSUPPORTED_SHAPE, "%s: K must be a multiple of 256", fn);
    if (N % 8) return fail(W2_ERR_UNSUPPORTED_SHAPE, "%s: N must be a multiple of 8", fn);
    if (K > (int64_t)1 << 24 || N > (int64_t)1 << 24)
        return fail(W2_ERR_UNSUPPORTED_SHAPE, "%s: K and N are limited to 2^24", fn);
    return W2_OK;
}

// Copies *t (NULL: all defaults) after checking every field against the values the header allows.
static int check_tuning(const char* fn, const w2_tuning_t* t, w2_tuning_t* out)
{
    memset(out, 0, sizeof *out);
    if (!t) return W2_OK;
    auto in = [](int v, int lo, int hi) { return v == 0 || (v >= lo && v <= hi); };
    auto one_of = [](int v, int a, int b, int c = 0, int d = 0, int e = 0) {
        return v == 0 || v == a || v == b || (c && v == c) || (d && v == d) || (e && v == e);
    };
    const char* bad = nullptr;
    if (t->variant < W2_VARIANT_AUTO || t->variant > W2_VARIANT_GEMV) bad = "variant";
    else if (!in(t->dot4_max_m, 1, 4)) bad = "dot4_max_m";
    else if (!in(t->midm_min_m, 1, 256)) bad = "midm_min_m";
    else if (!in(t->midm_max_m, 1, 256)) bad = "midm_max_m";
    else if (!in(t->small_waves, 1, 16)) bad = "small_waves";
    else if (!one_of(t->small_cbw, 1, 2, 4, 8, 16)) bad = "small_cbw";
    else if (t->small_kc < 0 || t->small_kc % TILE_K) bad = "small_kc";
    else if (!one_of(t->gemv_window, 2, 4, 8)) bad = "gemv_window";
    else if (!in(t->gemv_max_m, 1, 32)) bad = "gemv_max_m";
    else if (!one_of(t->midm_cbw, 2, 4, 8)) bad = "midm_cbw";
    else if (!one_of(t->tiled_bm, 64, 128)) bad = "tiled_bm";
    else if (!one_of(t->tiled_bn, 64, 128, 256)) bad = "tiled_bn";
    else if (!one_of(t->tiled_kw, 1, 2, 4)) bad = "tiled_kw";
    else if (!one_of(t->tiled_wd, 2, 8)) bad = "tiled_wd";
    else if (!in(t->tiled_group_m, 1, 1024)) bad = "tiled_group_m";
    else if (!in(t->splitk, 1, 16)) bad = "splitk";
    else if (!in(t->splitk_min_tiles, 1, 1024)) bad = "splitk_min_tiles";
    else if (!one_of(t->stream_unroll, 4, 8, 16)) bad = "stream_unroll";
    else if (!in(t->stream_blocks, 1, 65536)) bad = "stream_blocks";
    else if (!in(t->gemv_cbw, 1, 16)) bad = "gemv_cbw";
    else if (!in(t->gemv_ks, 1, 16)) bad = "gemv_ks";
    else if (!in(t->fused_rows, 1, 8)) bad = "fused_rows";
    if (bad) return fail(W2_ERR_INVALID_ARG, "%s: w2_tuning_t.%s is out of range", fn, bad);
    *out = *t;
    return W2_OK;
}

}  // namespace w2

using namespace w2;

extern "C" {

int w2_packed_size(int64_t K, int64_t N, int G, size_t* bytes)
{
    if (!bytes) return fail(W2_ERR_INVALID_ARG, "w2_packed_size: bytes is NULL");
    int rc = check_shape("w2_packed_size", K, N, G);
    if (rc) return rc;
    *bytes = make_layout(K, N, G).total_bytes;
    return W2_OK;
}

int w2_prepack(const uint8_t* codes_KN, const uint16_t* scales, int64_t K, int64_t N, int G,
               w2_codec_t codec, void* packed, size_t packed_bytes, int32_t* bad_codes,
               void* stream)
{
    int rc = check_shape("w2_prepack", K, N, G);
    if (rc) return rc;
    if (!codes_KN || !scales || !packed) return fail(W2_ERR_INVALID_ARG, "w2_prepack: NULL pointer");
    if (codec != W2_CODEC_INT2 && codec != W2_CODEC_TERNARY)
        return fail(W2_ERR_INVALID_ARG, "w2_prepack: unknown codec %d", (int)codec);
    if (!aligned16(packed)) return fail(W2_ERR_MISALIGNED, "w2_prepack: packed must be 16-byte aligned");
    const Layout L = make_layout(K, N, G);
    if (packed_bytes < L.total_bytes)
        return fail(W2_ERR_BUFFER_TOO_SMALL, "w2_prepack: packed_bytes %zu < %zu", packed_bytes, L.total_bytes);
    return launch_prepack(codes_KN, scales, L, (int)codec, packed, bad_codes, (hipStream_t)stream);
}

int w2_quantize_rows(const void* X, w2_dtype_t x_dtype, int64_t M, int64_t K, int64_t ldx, int G,
                     int8_t* xq, float* sx, int32_t* gsum, void* stream)
{
    if (M < 0 || K <= 0) return fail(W2_ERR_INVALID_ARG, "w2_quantize_rows: bad M or K");
    if (x_dtype != W2_DT_F32 && x_dtype != W2_DT_BF16)
        return fail(W2_ERR_INVALID_ARG, "w2_quantize_rows: unknown dtype %d", (int)x_dtype);
    if (K % TILE_K) return fail(W2_ERR_UNSUPPORTED_SHAPE, "w2_quantize_rows: K must be a multiple of 256");
    if (gsum && G != 64 && G != 128)
        return fail(W2_ERR_UNSUPPORTED_SHAPE, "w2_quantize_rows: G must be 64 or 128 when gsum is given");
    if (M > 0x7fffffff) return fail(W2_ERR_UNSUPPORTED_SHAPE, "w2_quantize_rows: M too large");
    if (M == 0) return W2_OK;
    if (!X || !xq || !sx) return fail(W2_ERR_INVALID_ARG, "w2_quantize_rows: NULL pointer");
    if (ldx < K || ldx % 8) return fail(W2_ERR_MISALIGNED, "w2_quantize_rows: ldx must be >= K and a multiple of 8");
    if (!aligned16(X) || !aligned16(xq)) return fail(W2_ERR_MISALIGNED, "w2_quantize_rows: X and xq must be 16-byte aligned");
    return launch_quantize(X, x_dtype == W2_DT_BF16, M, K, ldx, gsum ? G : 128, xq, sx, gsum,
                           (hipStream_t)stream);
}

static int a8_common(const char* fn, const void* packed, int64_t K, int64_t N, int G,
                     const int8_t* xq, const float* sx, int64_t M, uint16_t* Y, int64_t ldy,
                     int32_t* acc_out, void* workspace, size_t workspace_bytes, const w2_tuning_t* tune, void* stream,
                     const Epilogue& epi = Epilogue())
{
    int rc = check_shape(fn, K, N, G);
    if (rc) return rc;
    if (M < 0) return fail(W2_ERR_INVALID_ARG, "%s: M < 0", fn);
    rc = check_epilogue(fn, epi, N);
    if (rc) return rc;
    w2_tuning_t tn;
    rc = check_tuning(fn, tune, &tn);
    if (rc) return rc;
    int variant = tn.variant;
    const int64_t n_out = epi.act == ACT_SILU_MUL ? N / 2 : N;
    if (variant == W2_VARIANT_SCALED16)
        return fail(W2_ERR_INVALID_ARG, "%s: variant %d not available for w2a8", fn, variant);
    if (M == 0) return W2_OK;
    if (!packed || !xq) return fail(W2_ERR_INVALID_ARG, "%s: NULL pointer", fn);
    if (!acc_out && (!sx || !Y)) return fail(W2_ERR_INVALID_ARG, "%s: NULL pointer", fn);
    if (!aligned16(packed) || !aligned16(xq) || (Y && !aligned16(Y)))
        return fail(W2_ERR_MISALIGNED, "%s: packed, xq and Y must be 16-byte aligned", fn);
    if (!acc_out && (ldy < n_out || ldy % 8))
        return fail(W2_ERR_MISALIGNED, "%s: ldy must be >= the number of output columns and a multiple of 8", fn);
    if (M > ((int64_t)1 << 24)) return fail(W2_ERR_UNSUPPORTED_SHAPE, "%s: M is limited to 2^24", fn);
    const Layout L = make_layout(K, N, G);
    A8Args a;
    a.codes = (const uint32_t*)packed;
    a.scales = (const uint16_t*)((const char*)packed + L.codes_bytes);
    a.xq = xq; a.sx = sx; a.Y = Y; a.acc_out = acc_out;
    a.M = M; a.K = K; a.N = N; a.ldy = ldy;
    a.n_cb = L.n_cb; a.n_kt = L.n_kt; a.G = G;
    if (workspace && !aligned16(workspace))
        return fail(W2_ERR_MISALIGNED, "%s: workspace must be 16-byte aligned", fn);
    a.part = (float*)workspace;                              // split-K partial results, if the kernel wants them
    a.part_bytes = workspace ? workspace_bytes : 0;
    a.epi = epi;
    a.tune = tn;
    int fallback = W2_VARIANT_SMALLM;                        // where the decode kernel cannot hold the rows
    if (variant == W2_VARIANT_AUTO) {
        // measured: the MFMA form is at least as fast as dot4 from M = 1 on; the mid-M kernel (one
        // fma per accumulator in the dequant, rolling weight window; its time hardly grows with M)
        // overtakes the small-M one at M = 4 on wide or very deep projections and at M = 9 on narrow ones (few
        // column blocks: it then splits K four ways with a barrier pair per tile), and is faster
        // than the tiled one up to M = 64
        const int dot4_max = tn.dot4_max_m;
        const int midm_min = tn.midm_min_m ? tn.midm_min_m : (a.n_cb >= 384 || a.n_kt > 64) ? 4 : 9;
        // Upper end.  Two bands of 64 rows (up to M = 128) on the narrowest projections only (up to 4096
        // columns, where the tiled kernel has too few tiles: 4096 x 4096 at M = 128 10 against 14.7 us; with room
        // for split-K partial results the tiled kernel is the faster one there once K reaches 14336).  Wider:
        // 8192 x 8192 at M = 128 runs 23.5 us through the tiled kernel with K split inside its workgroups
        // against 33 in two bands, 4096 x 6144 15.0 against 18.7.  On wide projections (24576 columns and more)
        // the tiled kernel takes over at M = 33, where the mid-M kernel goes to four row tiles per wave and its
        // LDS operand reads bound it (4096 x 28672 at M = 48: 15.8 against 19.0 us; 5120 x 34816: 27 against 40).
        // Deep K (56 tiles and more) with room for split-K partial results: the tiled kernel, its K cut across
        // and inside workgroups, takes over at M = 33 (28672 x 8192 at M = 64: 31 against 34 us; 17408 x 5120 at
        // M = 33: 18.0 against 19.2), on the narrowest projections at M = 65 (14336 x 4096: 19.2 against 21.2).
        const bool deep_ws = a.part_bytes && a.n_kt >= 56;
        const int midm_max = tn.midm_max_m ? tn.midm_max_m
                           : a.n_cb <= 256 ? (deep_ws ? 64 : 128) : a.n_cb >= 1536 || deep_ws ? 32 : 64;
        fallback = M >= midm_min && M <= midm_max && a8_midm_supports(a) ? W2_VARIANT_MIDM
                 : a8_smallm_supports(a)                                   ? W2_VARIANT_SMALLM
                                                                           : W2_VARIANT_TILED;
        // The decode kernel keeps whole rows in local memory and reads the weights once, like the mid-M
        // kernel, without that kernel's barrier pair per 1024 k: measured faster up to 8 rows wherever the
        // rows fit (4096 x 28672 at M = 8: 7.4 against 10.1 us; 8192 x 8192: 5.9 against 7.8), and up to 16 rows
        // while two workgroups share a CU (rows of at most 64 to 68 KiB: 4096 x 28672 at M = 16 10.1 against
        // 10.5 us, 4096 x 6144 5.2 against 6.0) or the projection is narrow (8192 x 8192 at M = 16: 7.5 against
        // 9.4 us; 8192 x 10240 at M = 12 / 16: 11.6 / 11.7 against 12.6 / 12.8); wide projections with long rows
        // lose (8192 x 57344 at M = 12: 33 against 28 us).
        // Rows of more than 72 KiB leave room for one workgroup per CU only: then the grid must fit the chip
        // in one round (17408 x 5120 at M = 8, 320 workgroups: 15.3 against 10.4 us through the mid-M kernel;
        // 14336 x 4096, 256 workgroups: 6.4 against 8.1).
        const int64_t row_bytes = M * (K + 32);
        int gcbw = M > 12 ? 8 : 4;                              // (the decode kernel's rule for five rows and more)
        while (gcbw > 1 && (a.n_cb / gcbw < 192 || (a.n_kt + 8 / gcbw - 1) / (8 / gcbw) > 16)) gcbw >>= 1;
        const int64_t gemv_wgs = (a.n_cb + gcbw - 1) / gcbw;
        // (up to K = 8192 two rounds still win: 8192 x 10240 at M = 9 .. 16, 320 workgroups, 11.6 to 11.8 against 12.4 to 12.9)
        const bool one_round = row_bytes <= 72 * 1024 || gemv_wgs <= 256 || a.n_kt <= 32;
        // narrow: few column blocks, or a grid of one round (8192 x 12288 at M = 9 .. 16, 192 workgroups: 9.1 to 9.3
        // against 12.8 to 13.2)
        const bool narrow = a.n_cb <= 640 || gemv_wgs <= 256;
        const int gemv_max = tn.gemv_max_m                               ? tn.gemv_max_m
                           : M <= 4                                      ? 4
                           : !one_round                                  ? 4
                           : M <= 8                                      ? 8
                           : M <= 12 && (row_bytes <= 64 * 1024 || narrow) ? 12
                           : M <= 16 ? (row_bytes <= 68 * 1024 || narrow ? 16 : 8)
                           // 17 to 32 rows (two row tiles per wave, one workgroup per CU): K up to 4096 in a grid of
                           // one round (4096 x 4096 at M = 17..32: 5.9 against 6.9 to 7.3 us through the mid-M
                           // kernel; 4096 x 6144 6.8 against 7.2; 4096 x 28672 12.5 to 13.9 against 13.0 to 14.3;
                           // K = 5120 gains nothing, 4096 x 57344, two rounds, loses 10 %)
                           : M <= 32 && a.n_kt <= 16 && row_bytes <= 133 * 1024 ? 32
                                                                         : 8;
        variant = M <= dot4_max && a8_dot4_supports(a)     ? W2_VARIANT_DOT4
                : M <= gemv_max && a8_gemv_supports(M)     ? W2_VARIANT_GEMV
                                                           : fallback;
    }
    hipStream_t s = (hipStream_t)stream;
    switch (variant) {
    case W2_VARIANT_GEMV: {
        if (!a8_gemv_supports(M)) return fail(W2_ERR_UNSUPPORTED_SHAPE, "%s: GEMV needs M <= 32", fn);
        rc = launch_a8_gemv(a, xq, 0, K, s);
        // rows too long for one workgroup's local memory: the kernels that stage them in chunks
        if (rc != W2_ERR_UNSUPPORTED_SHAPE || tn.variant == W2_VARIANT_GEMV) return rc;
        if (fallback == W2_VARIANT_MIDM) return launch_a8_midm(a, s);
        if (fallback == W2_VARIANT_TILED) return launch_a8_tiled(a, s);
        return launch_a8_smallm(a, s);
    }
    case W2_VARIANT_DOT4:
        if (!a8_dot4_supports(a)) return fail(W2_ERR_UNSUPPORTED_SHAPE, "%s: DOT4 needs M <= 4", fn);
        return launch_a8_dot4(a, s);
    case W2_VARIANT_SMALLM:
        if (!a8_smallm_supports(a)) return fail(W2_ERR_UNSUPPORTED_SHAPE, "%s: SMALLM needs M <= 16", fn);
        return launch_a8_smallm(a, s);
    case W2_VARIANT_MIDM:
        if (!a8_midm_supports(a)) return fail(W2_ERR_UNSUPPORTED_SHAPE, "%s: MIDM needs M <= 256", fn);
        return launch_a8_midm(a, s);
    default:
        return launch_a8_tiled(a, s);
    }
}

int w2_matmul_a8_ex(const void* packed, int64_t K, int64_t N, int G, const int8_t* xq,
                    const float* sx, int64_t M, uint16_t* Y, int64_t ldy, void* workspace,
                    size_t workspace_bytes, const w2_tuning_t* tune, void* stream)
{
    return a8_common("w2_matmul_a8", packed, K, N, G, xq, sx, M, Y, ldy, nullptr, workspace, workspace_bytes, tune,
                     stream);
}

int w2_matmul_a8(const void* packed, int64_t K, int64_t N, int G, const int8_t* xq,
                 const float* sx, int64_t M, uint16_t* Y, int64_t ldy, void* workspace,
                 size_t workspace_bytes, void* stream)
{
    return w2_matmul_a8_ex(packed, K, N, G, xq, sx, M, Y, ldy, workspace, workspace_bytes, nullptr, stream);
}

// Workspace that lets w2_matmul_a8_fused take the two-kernel route: int8 rows + one scale per row
// (rounded up to 256 bytes: split-K partial results may follow).
static size_t fused_workspace_bytes(int64_t M, int64_t K)
{
    return ((size_t)((M * K + 15) & ~(int64_t)15) + (size_t)M * sizeof(float) + 255) & ~(size_t)255;
}

static int a8_fused_common(const char* fn, const void* packed, int64_t K, int64_t N, int G, const void* X,
                           w2_dtype_t x_dtype, int64_t ldx, int64_t M, uint16_t* Y, int64_t ldy,
                           void* workspace, size_t workspace_bytes, const w2_tuning_t* tune, void* stream,
                           const Epilogue& epi)
{
    int rc = check_shape(fn, K, N, G);
    if (rc) return rc;
    rc = check_epilogue(fn, epi, N);
    if (rc) return rc;
    w2_tuning_t tn;
    rc = check_tuning(fn, tune, &tn);
    if (rc) return rc;
    const int64_t n_out = epi.act == ACT_SILU_MUL ? N / 2 : N;
    if (M < 0) return fail(W2_ERR_INVALID_ARG, "%s: M < 0", fn);
    if (x_dtype != W2_DT_F32 && x_dtype != W2_DT_BF16)
        return fail(W2_ERR_INVALID_ARG, "%s: unknown dtype %d", fn, (int)x_dtype);
    if (M == 0) return W2_OK;
    if (!packed || !X || !Y) return fail(W2_ERR_INVALID_ARG, "%s: NULL pointer", fn);
    if (!aligned16(packed) || !aligned16(X) || !aligned16(Y))
        return fail(W2_ERR_MISALIGNED, "%s: packed, X and Y must be 16-byte aligned", fn);
    if (ldx < K || ldx % 8 || ldy < n_out || ldy % 8)
        return fail(W2_ERR_MISALIGNED, "%s: ldx >= K, ldy >= the number of output columns, both multiples of 8", fn);
    if (workspace && !aligned16(workspace))
        return fail(W2_ERR_MISALIGNED, "%s: workspace must be 16-byte aligned", fn);
    const Layout L = make_layout(K, N, G);
    // Measured: one launch with the abs-max reduced per workgroup is at least as fast as quantise + matmul
    // up to four rows wherever a workgroup can hold the rows (4096 x 28672 at M = 4: 10.2 against 11.0 us,
    // 4096 x 4096: 5.3 against 6.3), and up to eight rows (the wide form) while a thread stages one piece per
    // row, K <= 4096 (M = 8, bf16 rows: 4096 x 28672 10.7 against 11.8 us, 4096 x 4096 5.0 against 6.6; at
    // K = 5120 5120 x 34816 23.8 against 14.1); beyond, every workgroup re-reading and re-quantising all rows
    // costs more than a separate quantise launch (the paper's finding for multi-row activations, Sec. III-C:
    // twelve rows of 4096 x 6144 8.2 against 7.7 us).
    const bool ws_ok = workspace && workspace_bytes >= fused_workspace_bytes(M, K);
    const int one_launch_rows = tn.fused_rows ? tn.fused_rows : K <= 4096 ? 8 : 4;
    if (M > 4 && !ws_ok) {
        if (workspace)
            return fail(W2_ERR_BUFFER_TOO_SMALL, "%s: M = %lld needs a workspace of %zu bytes (w2_workspace_size)",
                        fn, (long long)M, fused_workspace_bytes(M, K));
        return fail(W2_ERR_UNSUPPORTED_SHAPE, "%s: M = %lld needs a workspace (w2_workspace_size)", fn, (long long)M);
    }
    if (M <= one_launch_rows || !ws_ok) {
        A8Args a;
        a.codes = (const uint32_t*)packed;
        a.scales = (const uint16_t*)((const char*)packed + L.codes_bytes);
        a.xq = nullptr; a.sx = nullptr; a.Y = Y; a.acc_out = nullptr;
        a.M = M; a.K = K; a.N = N; a.ldy = ldy; a.n_cb = L.n_cb; a.n_kt = L.n_kt; a.G = G;
        a.epi = epi; a.tune = tn;
        rc = launch_a8_gemv(a, X, x_dtype == W2_DT_BF16 ? 2 : 1, ldx, (hipStream_t)stream);
        if (rc != W2_ERR_UNSUPPORTED_SHAPE || !ws_ok) return rc;
    }
    int8_t* xq = (int8_t*)workspace;
    float* sx = (float*)((char*)workspace + ((M * K + 15) & ~(int64_t)15));
    rc = launch_quantize(X, x_dtype == W2_DT_BF16, M, K, ldx, G, xq, sx, nullptr, (hipStream_t)stream);
    if (rc) return rc;
    const size_t used = fused_workspace_bytes(M, K);
    return a8_common(fn, packed, K, N, G, xq, sx, M, Y, ldy, nullptr, (char*)workspace + used, workspace_bytes - used,
                     tune, stream, epi);
}

static Epilogue to_epilogue(const w2_epilogue_t* e)
{
    Epilogue r;
    if (e) { r.bias = e->bias; r.act = e->act; }
    return r;
}

int w2_matmul_a8_fused(const void* packed, int64_t K, int64_t N, int G, const void* X,
                       w2_dtype_t x_dtype, int64_t ldx, int64_t M, uint16_t* Y, int64_t ldy,
                       void* workspace, size_t workspace_bytes, void* stream)
{
    return a8_fused_common("w2_matmul_a8_fused", packed, K, N, G, X, x_dtype, ldx, M, Y, ldy, workspace,
                           workspace_bytes, nullptr, stream, Epilogue());
}

// ---- the entry point that allocates nothing -------------------------------------------------
// The scratch memory w2_matmul_a8_fused otherwise takes from the caller's workspace (the int8 rows,
// their scales, split-K partial results) lives in this array: device memory that exists from the
// moment the library's code object is loaded on a GPU until the process ends, one copy per GPU.
// In host code the array's name is only a handle for hipGetSymbolAddress; the address it returns
// (per device) is what kernels and copies get.
constexpr size_t W2_SCRATCH_BYTES = (size_t)W2_NOALLOC_SCRATCH_MIB << 20;
static __device__ __align__(256) unsigned char scratch[W2_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[MAX_DEVICES] = {};
}  // namespace

// Device address of `scratch` on the current device, resolved once per device.
static int scratch_address(const char* fn, void** out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(W2_ERR_HIP, "%s: hipGetDevice: %s", fn, hipGetErrorString(e));
    if (dev < 0 || dev >= MAX_DEVICES) return fail(W2_ERR_HIP, "%s: device ordinal %d not supported", fn, dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return fail(W2_ERR_HIP, "%s: hipGetSymbolAddress(scratch): %s", fn, hipGetErrorString(e));
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return W2_OK;
}

int w2_init(void)
{
    void* p;
    return scratch_address("w2_init", &p);
}

int w2_matmul_a8_fused_noalloc(const void* packed, int64_t K, int64_t N, int G, const void* X,
                               w2_dtype_t x_dtype, int64_t ldx, int64_t M, uint16_t* Y, int64_t ldy,
                               void* stream)
{
    const char* fn = "w2_matmul_a8_fused_noalloc";
    int rc = check_shape(fn, K, N, G);
    if (rc) return rc;
    if (M < 0) return fail(W2_ERR_INVALID_ARG, "%s: M < 0", fn);
    if (M > ((int64_t)1 << 24)) return fail(W2_ERR_UNSUPPORTED_SHAPE, "%s: M is limited to 2^24", fn);
    // the quantised rows and their scales must fit the built-in scratch (what is left goes to split-K)
    const size_t need = M > 0 ? fused_workspace_bytes(M, K) : 0;
    if (need > W2_SCRATCH_BYTES)
        return fail(W2_ERR_BUFFER_TOO_SMALL,
                    "%s: M*K = %lld needs %zu bytes of scratch, the built-in buffer holds %zu "
                    "(use w2_matmul_a8_fused with a workspace)", fn, (long long)(M * K), need, W2_SCRATCH_BYTES);
    void* ws = nullptr;
    rc = scratch_address(fn, &ws);
    if (rc) return rc;
    return a8_fused_common(fn, packed, K, N, G, X, x_dtype, ldx, M, Y, ldy, ws, W2_SCRATCH_BYTES, nullptr, stream,
                           Epilogue());
}

int w2_matmul_a8_fused_epi(const void* packed, int64_t K, int64_t N, int G, const void* X,
                           w2_dtype_t x_dtype, int64_t ldx, int64_t M, uint16_t* Y, int64_t ldy,
                           const w2_epilogue_t* epi, void* workspace, size_t workspace_bytes,
                           const w2_tuning_t* tune, void* stream)
{
    return a8_fused_common("w2_matmul_a8_fused_epi", packed, K, N, G, X, x_dtype, ldx, M, Y, ldy, workspace,
                           workspace_bytes, tune, stream, to_epilogue(epi));
}

int w2_matmul_a8_epi(const void* packed, int64_t K, int64_t N, int G, const int8_t* xq, const float* sx,
                     int64_t M, uint16_t* Y, int64_t ldy, const w2_epilogue_t* epi, void* workspace,
                     size_t workspace_bytes, const w2_tuning_t* tune, void* stream)
{
    return a8_common("w2_matmul_a8_epi", packed, K, N, G, xq, sx, M, Y, ldy, nullptr, workspace, workspace_bytes,
                     tune, stream, to_epilogue(epi));
}

int w2_debug_group_acc_a8(const void* packed, int64_t K, int64_t N, int G, const int8_t* xq,
                          int64_t M, const w2_tuning_t* tune, int32_t* acc, void* stream)
{
    if (!acc && M > 0) return fail(W2_ERR_INVALID_ARG, "w2_debug_group_acc_a8: acc is NULL");
    return a8_common("w2_debug_group_acc_a8", packed, K, N, G, xq, nullptr, M, nullptr, 0, acc, nullptr, 0,
                     tune, stream);
}

static int a16_common(const char* fn, const void* packed, int64_t K, int64_t N, int G,
                      const uint16_t* X, int64_t ldx, int64_t M, uint16_t* Y, int64_t ldy,
                      void* workspace, size_t workspace_bytes, const w2_tuning_t* tune, void* stream,
                      const Epilogue& epi = Epilogue())
{
    int rc = check_shape(fn, K, N, G);
    if (rc) return rc;
    if (M < 0) return fail(W2_ERR_INVALID_ARG, "%s: M < 0", fn);
    rc = check_epilogue(fn, epi, N);
    if (rc) return rc;
    w2_tuning_t tn;
    rc = check_tuning(fn, tune, &tn);
    if (rc) return rc;
    int variant = tn.variant;
    const int64_t n_out = epi.act == ACT_SILU_MUL ? N / 2 : N;
    if (variant != W2_VARIANT_AUTO && variant != W2_VARIANT_SMALLM && variant != W2_VARIANT_TILED &&
        variant != W2_VARIANT_SCALED16 && variant != W2_VARIANT_MIDM && variant != W2_VARIANT_GEMV)
        return fail(W2_ERR_INVALID_ARG, "%s: variant %d not available for w2a16", fn, variant);
    if (M == 0) return W2_OK;
    if (!packed || !X || !Y) return fail(W2_ERR_INVALID_ARG, "%s: NULL pointer", fn);
    if (!aligned16(packed) || !aligned16(X) || !aligned16(Y))
        return fail(W2_ERR_MISALIGNED, "%s: packed, X and Y must be 16-byte aligned", fn);
    if (ldx < K || ldx % 8 || ldy < n_out || ldy % 8)
        return fail(W2_ERR_MISALIGNED, "%s: ldx >= K, ldy >= the number of output columns, both multiples of 8", fn);
    if (M > ((int64_t)1 << 24)) return fail(W2_ERR_UNSUPPORTED_SHAPE, "%s: M is limited to 2^24", fn);
    // the tiled kernel addresses a workgroup's 64 rows with 32-bit byte offsets
    if (ldx > ((int64_t)1 << 24)) return fail(W2_ERR_UNSUPPORTED_SHAPE, "%s: ldx is limited to 2^24", fn);
    const Layout L = make_layout(K, N, G);
    A16Args a;
    a.codes = (const uint32_t*)packed;
    a.scales = (const uint16_t*)((const char*)packed + L.codes_bytes);
    a.X = X; a.Y = Y; a.M = M; a.K = K; a.N = N; a.ldx = ldx; a.ldy = ldy;
    a.n_cb = L.n_cb; a.n_kt = L.n_kt; a.G = G;
    if (workspace && !aligned16(workspace))
        return fail(W2_ERR_MISALIGNED, "%s: workspace must be 16-byte aligned", fn);
    a.part = (float*)workspace;                              // split-K partial results, if the kernel wants them
    a.part_bytes = workspace ? workspace_bytes : 0;
    a.epi = epi;
    a.tune = tn;
    a.fold = variant == W2_VARIANT_SCALED16;
    if (variant == W2_VARIANT_GEMV) return launch_a16_gemv(a, (hipStream_t)stream);
    if (variant == W2_VARIANT_SCALED16) {
        // the scale-folded construction: the small-M kernel with it, or the kernels built on it
        if (!a16_smallm_supports(a))
            return M <= 64 ? launch_a16_midm(a, (hipStream_t)stream) : launch_a16_fold_tiled(a, (hipStream_t)stream);
        variant = W2_VARIANT_SMALLM;
    }
    if (variant == W2_VARIANT_AUTO) {
        // Few rows: the decode kernel (below), else the zero-point construction in the small-M kernel; up to
        // 64 rows the mid-M kernel (the weight stream is still read once; measured faster than the small-M
        // kernel from M = 9 on every projection shape); above, 128-row tiles.  Both of the latter fold the
        // scale into the weights: fewest vector instructions per matrix instruction.
        // (K beyond 16384: from M = 3, for the rows the decode kernel cannot hold; 17408 x 5120 at M = 8 19.9 us
        // against 33.7 in the small-M kernel, at M = 4 19.2 against 25.5)
        // (with room for split-K partial results already from K = 8448 on: 14336 x 4096 at M = 8 13.8 us against 15.4)
        // (and on the widest projections once K passes 5120, where five to eight rows leave the decode kernel one
        // workgroup per CU: 8192 x 57344 at M = 5 / 8 42.3 / 43.1 us against 43.7 / 45.8)
        const bool wide_deep = K > 5120 && a.n_cb >= 2048;
        const int midm_min = tn.midm_min_m ? tn.midm_min_m
                           : a.n_kt > 64 ? 3 : (a.n_kt > 32 && a.part_bytes) || wide_deep ? 5 : 9;
        // two bands on small projections; on very wide ones (32768 columns and more) the tiled kernel
        // takes over at M = 41 (8192 x 57344 at M = 48: 94 against 104 us)
        // (and with room for split-K partial results the tiled kernel wins above 64 rows once K passes 8192:
        // 28 against 35 us on 14336 x 4096 at M = 128)
        const int midm_max = tn.midm_max_m ? tn.midm_max_m
                           : a.n_cb <= 256 ? (a.part_bytes && a.n_kt > 32 ? 64 : 128) : a.n_cb >= 2048 ? 40 : 64;
        // The decode kernel wherever a workgroup can hold the rows: up to 8 of them, and up to 16 while a thread
        // stages one piece per row (K <= 4096: 4096 x 28672 at M = 12 14.0 us against 15.9 in the mid-M kernel,
        // 4096 x 4096 6.4 against 7.6; 5120 x 34816 31 against 29)
        const bool gemv_rows = tn.midm_min_m ? M < midm_min : M <= 4 || (M <= 8 && !wide_deep) || (M <= 16 && K <= 4096);
        if (gemv_rows && a16_gemv_supports(a)) {
            rc = launch_a16_gemv(a, (hipStream_t)stream);
            if (rc != W2_ERR_UNSUPPORTED_SHAPE) return rc;   // (a shape it turns down after all goes on to the other kernels)
        }
        if (M >= midm_min && M <= midm_max && a16_midm_supports(a)) return launch_a16_midm(a, (hipStream_t)stream);
        if (a16_gemv_supports(a)) {
            rc = launch_a16_gemv(a, (hipStream_t)stream);
            if (rc != W2_ERR_UNSUPPORTED_SHAPE) return rc;   // (a shape it turns down after all goes on to the small-M kernel)
        }
        if (!a16_smallm_supports(a)) return launch_a16_fold_tiled(a, (hipStream_t)stream);
        variant = W2_VARIANT_SMALLM;
    }
    if (variant == W2_VARIANT_MIDM) {
        if (!a16_midm_supports(a)) return fail(W2_ERR_UNSUPPORTED_SHAPE, "%s: MIDM needs M <= 256", fn);
        return launch_a16_midm(a, (hipStream_t)stream);
    }
    if (variant == W2_VARIANT_SMALLM) {
        if (!a16_smallm_supports(a)) return fail(W2_ERR_UNSUPPORTED_SHAPE, "%s: SMALLM needs M <= 16", fn);
        return launch_a16_smallm(a, (hipStream_t)stream);
    }
    return launch_a16_tiled(a, (hipStream_t)stream);
}

int w2_matmul_a16_ex(const void* packed, int64_t K, int64_t N, int G, const uint16_t* X,
                     int64_t ldx, int64_t M, uint16_t* Y, int64_t ldy, void* workspace,
                     size_t workspace_bytes, const w2_tuning_t* tune, void* stream)
{
    return a16_common("w2_matmul_a16", packed, K, N, G, X, ldx, M, Y, ldy, workspace, workspace_bytes, tune,
                      stream);
}

int w2_matmul_a16_epi(const void* packed, int64_t K, int64_t N, int G, const uint16_t* X, int64_t ldx, int64_t M,
                      uint16_t* Y, int64_t ldy, const w2_epilogue_t* epi, void* workspace, size_t workspace_bytes,
                      const w2_tuning_t* tune, void* stream)
{
    return a16_common("w2_matmul_a16_epi", packed, K, N, G, X, ldx, M, Y, ldy, workspace, workspace_bytes, tune,
                      stream, to_epilogue(epi));
}

int w2_matmul_a16(const void* packed, int64_t K, int64_t N, int G, const uint16_t* X,
                  int64_t ldx, int64_t M, uint16_t* Y, int64_t ldy, void* workspace,
                  size_t workspace_bytes, void* stream)
{
    return w2_matmul_a16_ex(packed, K, N, G, X, ldx, M, Y, ldy, workspace, workspace_bytes, nullptr, stream);
}

int w2_workspace_size(int64_t M, int64_t K, int64_t N, int G, int a16, size_t* bytes)
{
    if (!bytes) return fail(W2_ERR_INVALID_ARG, "w2_workspace_size: bytes is NULL");
    int rc = check_shape("w2_workspace_size", K, N, G);
    if (rc) return rc;
    if (M < 0) return fail(W2_ERR_INVALID_ARG, "w2_workspace_size: M < 0");
    // one or two rows of up to 64 KiB (as fp32) run as a single launch and need none
    const bool single = M <= 2 && M * K * 4 <= 64 * 1024;
    const Layout L = make_layout(K, N, G);
    const w2_tuning_t dflt = {};
    if (M == 0) *bytes = 0;
    else if (a16) {
        const size_t tiled = M > 64 ? a16_fold_splitk_bytes(M, N, L.n_kt, dflt) : 0;
        const size_t midm = M >= 3 && M <= 128 ? a16_midm_splitk_bytes(M, N, L.n_cb, L.n_kt, dflt) : 0;
        *bytes = tiled > midm ? tiled : midm;
    }
    else {
        // split-K partial results: the tiled kernel's above 64 rows, the mid-M kernel's on deep projections
        // (whichever of the two the call would pick, the larger need covers it)
        const size_t tiled = M > 32 ? a8_tiled_splitk_bytes(M, N, L.n_kt, G, dflt) : 0;
        const size_t midm = M >= 4 && M <= 128 ? a8_midm_splitk_bytes(M, N, L.n_cb, L.n_kt, dflt) : 0;
        *bytes = (single ? 0 : fused_workspace_bytes(M, K)) + (tiled > midm ? tiled : midm);
    }
    return W2_OK;
}

int w2_debug_unpack(const void* packed, int64_t K, int64_t N, int G, w2_codec_t codec,
                    uint8_t* codes_KN, uint16_t* scales, void* stream)
{
    int rc = check_shape("w2_debug_unpack", K, N, G);
    if (rc) return rc;
    if (!packed || !codes_KN || !scales) return fail(W2_ERR_INVALID_ARG, "w2_debug_unpack: NULL pointer");
    if (codec != W2_CODEC_INT2 && codec != W2_CODEC_TERNARY)
        return fail(W2_ERR_INVALID_ARG, "w2_debug_unpack: unknown codec %d", (int)codec);
    return launch_unpack(packed, make_layout(K, N, G), (int)codec, codes_KN, scales,
                         (hipStream_t)stream);
}

int w2_debug_stream_read(const void* src, size_t bytes, uint32_t* sink, const w2_tuning_t* tune, void* stream)
{
    if (!src || !sink) return fail(W2_ERR_INVALID_ARG, "w2_debug_stream_read: NULL pointer");
    if (!aligned16(src)) return fail(W2_ERR_MISALIGNED, "w2_debug_stream_read: src must be 16-byte aligned");
    w2_tuning_t tn;
    const int rc = check_tuning("w2_debug_stream_read", tune, &tn);
    if (rc) return rc;
    return launch_stream_read(src, bytes, sink, tn, (hipStream_t)stream);
}

int w2_debug_int8_gemv(const int8_t* W8, int64_t K, int64_t N, const int8_t* xq, int32_t* out, void* stream)
{
    if (K <= 0 || N <= 0) return fail(W2_ERR_INVALID_ARG, "w2_debug_int8_gemv: K and N must be positive");
    if (K % 16 || K > 49152) return fail(W2_ERR_UNSUPPORTED_SHAPE, "w2_debug_int8_gemv: K must be a multiple of 16, at most 49152");
    if (N > (int64_t)1 << 24) return fail(W2_ERR_UNSUPPORTED_SHAPE, "w2_debug_int8_gemv: N is limited to 2^24");
    if (!W8 || !xq || !out) return fail(W2_ERR_INVALID_ARG, "w2_debug_int8_gemv: NULL pointer");
    if (!aligned16(W8) || !aligned16(xq)) return fail(W2_ERR_MISALIGNED, "w2_debug_int8_gemv: W8 and xq must be 16-byte aligned");
    return launch_int8_gemv(W8, xq, out, K, N, (hipStream_t)stream);
}

const char* w2_status_string(int status)
{
    switch (status) {
    case W2_OK: return "ok";
    case W2_ERR_INVALID_ARG: return "invalid argument";
    case W2_ERR_UNSUPPORTED_SHAPE: return "unsupported shape";
    case W2_ERR_MISALIGNED: return "misaligned pointer or stride";
    case W2_ERR_BUFFER_TOO_SMALL: return "buffer too small";
    case W2_ERR_HIP: return "HIP error";
    case W2_ERR_BAD_CODE: return "weight code outside the codec's alphabet";
    default: return "unknown status";
    }
}

const char* w2_last_error(void) { return g_err; }

}  // extern "C"
