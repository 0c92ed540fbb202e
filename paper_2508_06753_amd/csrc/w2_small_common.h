// Pieces shared by the small-M kernels (w2a8 and w2a16): the streamed tile
// registers, the per-wave schedule and the launch configuration.
#pragma once
#include <hip/hip_runtime.h>

#include "w2_internal.h"

namespace w2 {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int XS_PAD = 32;   // bytes of padding per LDS activation row: a row stride of 32 mod 64 bytes spreads the MFMA A-operand reads over all banks

__device__ __forceinline__ float bf16_to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// two fp32 -> two bf16 (round to nearest even) in one dword, lo in the low half: one conversion instruction
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// x * sigmoid(x); v_exp_f32 and v_rcp_f32 are good to about 1e-6 relative, far inside a bf16 result
__device__ __forceinline__ float silu_f32(float z) { return z * __frcp_rn(1.0f + __expf(-z)); }

// The store loop shared by the kernels that reduce their k-splits through LDS: a workgroup holds
// `cbw` adjacent column blocks starting at block first_cb, `rows` rows; z(ci, m, nl) returns the
// finished fp32 result of column block ci, row m, column nl of the block.  Applies the fused
// epilogue; for the gated form cbw and first_cb are even and a thread combines a gate and an up
// column.
template <typename ZFn>
__device__ __forceinline__ void store_outputs(const Epilogue& e, uint16_t* __restrict__ Y, int64_t ldy, int64_t N,
                                              int64_t first_cb, int cbw, int rows, ZFn z)
{
    if (e.act != ACT_SILU_MUL) {
        const int outs = cbw * rows * 16;
        for (int i = threadIdx.x; i < outs; i += blockDim.x) {
            const int nl = i & 15, m = (i >> 4) % rows, ci = i / (16 * rows);
            const int64_t nn = (first_cb + ci) * TILE_N + nl;
            if (nn >= N) continue;
            float v = z(ci, m, nl, i);
            if (e.bias) v += bf16_to_f32(e.bias[nn]);
            if (e.act == ACT_SILU) v = silu_f32(v);
            Y[(int64_t)m * ldy + nn] = f32_to_bf16_rne(v);
        }
    } else {
        const int outs = (cbw >> 1) * rows * 16;
        for (int i = threadIdx.x; i < outs; i += blockDim.x) {
            const int nl = i & 15, m = (i >> 4) % rows, p = i / (16 * rows);
            const int64_t ng = (first_cb + 2 * p) * TILE_N + nl, nu = ng + TILE_N;
            if (nu >= N) continue;                           // N % 32 == 0: both or neither
            float g = z(2 * p, m, nl, i), u = z(2 * p + 1, m, nl, i);
            if (e.bias) {
                g += bf16_to_f32(e.bias[ng]);
                u += bf16_to_f32(e.bias[nu]);
            }
            Y[(int64_t)m * ldy + ((first_cb >> 1) + p) * TILE_N + nl] = f32_to_bf16_rne(silu_f32(g) * u);
        }
    }
}

// 16 two-bit fields -> four dwords of int8 lanes holding 64*q.
__device__ __forceinline__ void upconvert(uint32_t w, int (&u)[4])
{
    u[0] = (int)((w << 6) & 0xC0C0C0C0u);
    u[1] = (int)((w << 4) & 0xC0C0C0C0u);
    u[2] = (int)((w << 2) & 0xC0C0C0C0u);
    u[3] = (int)(w & 0xC0C0C0C0u);
}

// One streamed tile: 16 B of codes and the tile's group scales for this lane.
struct TileRegs {
    uint4 w;
    uint32_t s0, s1;   // bf16 scales: G=128 -> s0 = {g0,g1}; G=64 -> s0 = {g0,g1}, s1 = {g2,g3}
};

template <int G>
__device__ __forceinline__ TileRegs load_tile(const uint32_t* __restrict__ codes,
                                              const uint16_t* __restrict__ scales, int64_t tile,
                                              int lane)
{
    TileRegs r;
    // non-temporal: the weights are streamed once and should not displace anything in the caches
    // (measured: the plain streaming read gains 10 % from the hint, the GEMV kernels 1-3 %)
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(codes + (tile * 64 + lane) * 4));
    r.w = make_uint4(t[0], t[1], t[2], t[3]);
    if constexpr (G == 128) {
        r.s0 = *reinterpret_cast<const uint32_t*>(scales + (tile * TILE_N + (lane & 15)) * 2);
        r.s1 = 0;
    } else {
        const uint2 s = *reinterpret_cast<const uint2*>(scales + (tile * TILE_N + (lane & 15)) * 4);
        r.s0 = s.x; r.s1 = s.y;
    }
    return r;
}

template <int G>
__device__ __forceinline__ float tile_scale(const TileRegs& r, int gi)
{
    // gi = group index inside the tile
    const uint32_t pair = (G == 128 || gi < 2) ? r.s0 : r.s1;
    return (gi & 1) ? __uint_as_float(pair & 0xffff0000u) : __uint_as_float(pair << 16);
}

struct SmallCfg {
    int cbw;        // column blocks per workgroup
    int ks;         // k-splits inside the workgroup (waves = cbw * ks)
    int kc;         // k per LDS chunk (multiple of 256)
};

// The per-wave schedule shared by both kernel families.  A wave owns column
// block cb and the k tiles ks, ks+KS, ...  Inside one LDS chunk it first issues
// the loads of ALL its tiles (up to TMAX, 1 KiB each per wave) and only then
// consumes them, so a wave has its whole share of the weight stream in flight
// after one round trip: the kernels live for a few microseconds, about as long
// as a handful of dependent HBM round trips.
#define W2_SMALL_PROLOGUE()                                                                   \
    extern __shared__ __align__(16) int8_t smem[];                                            \
    const int lane = threadIdx.x & 63;                                                        \
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);                        \
    const int cbi = wave % cfg.cbw;                                                           \
    const int ks = wave / cfg.cbw;                                                            \
    const int64_t cb = (int64_t)blockIdx.x * cfg.cbw + cbi;                                   \
    const bool cb_ok = cb < a.n_cb;                                                           \
    const int64_t cbc = cb_ok ? cb : a.n_cb - 1; /* clamp: keeps loads in bounds */           \
    const int q = lane >> 4;                                                                  \
    const int64_t n = cb * TILE_N + (lane & 15);                                              \
    constexpr int GPT = TILE_K / G;                                                           \
    const int tiles_per_chunk = cfg.kc / TILE_K;                                              \
    const int n_chunks = (int)((a.n_kt + tiles_per_chunk - 1) / tiles_per_chunk);             \
    (void)n; (void)q; (void)GPT


// ---------------------------------------------------------------- host side

constexpr int TMAX = 8;                      // most tiles a wave keeps in flight
constexpr int64_t LDS_BUDGET = 128 * 1024;   // activation chunk + reduction scratch

// Picks (column blocks per workgroup, k-splits): enough workgroups to fill 256
// CUs a few times over, and a k-split that leaves each wave at most TMAX tiles
// when the wave budget allows it.  Eight waves per workgroup, or four when eight
// would make more than 512 workgroups (a CU holds about two eight-wave
// workgroups of these kernels at a time; on wide projections the finer grain
// fills the chip better: measured 13.5 against 15.6 us on 5120 x 34816 and 26.1
// against 29.7 us on 8192 x 57344 at M = 1, no change on 4096 x 28672).
static SmallCfg pick_cfg(const w2_tuning_t& tune, int64_t n_cb, int64_t n_kt, int rows, int bytes_per_k,
                         int max_waves = 16, bool even_cbw = false, int min_threads = 0)
{
    SmallCfg c;
    int waves = tune.small_waves;                            // validated by the entry point: 0 or 1..16
    const bool auto_waves = waves <= 0;
    if (auto_waves) waves = 8;
    if (waves > max_waves) waves = max_waves;
    if (waves < 1) waves = 1;
    const int cbw_env = tune.small_cbw;                      // 0 or a power of two <= 16
    auto choose = [&](int w) {
        int cb = w;
        // split K until a wave has at most TMAX tiles, while there are waves to split over
        while (cb > 1 && n_kt * cb > (int64_t)TMAX * w) cb >>= 1;
        // and keep at least one workgroup per CU
        while (cb > 1 && (n_cb + cb - 1) / cb < 256) cb >>= 1;
        return cb;
    };
    int cbw = cbw_env > 0 ? cbw_env : choose(waves);
    if (auto_waves && cbw_env <= 0 && waves == 8 && (n_cb + cbw - 1) / cbw > 512 && 4 * 64 >= min_threads) {
        waves = 4;
        cbw = choose(waves);
    }
    if (cbw > waves) cbw = waves;
    if (even_cbw && (cbw & 1)) cbw = cbw == 1 ? 2 : cbw - 1;     // the gated epilogue pairs adjacent column blocks
    c.cbw = cbw;
    c.ks = waves / cbw;
    if (c.ks > n_kt) c.ks = (int)n_kt;
    if (c.ks < 1) c.ks = 1;
    int64_t kc = n_kt * TILE_K;
    while (kc > TILE_K && (int64_t)rows * (kc * bytes_per_k + XS_PAD) > LDS_BUDGET) kc -= TILE_K;
    const int force = tune.small_kc;
    if (force >= TILE_K && force % TILE_K == 0 && force < kc) kc = force;
    c.kc = (int)kc;
    return c;
}

static size_t small_lds_bytes(const SmallCfg& c, int rows, int red_rows, int bytes_per_k, size_t extra)
{
    size_t act = (size_t)rows * (c.kc * bytes_per_k + XS_PAD) + extra;
    size_t red = (size_t)c.cbw * c.ks * red_rows * 16 * sizeof(float);
    return act > red ? act : red;
}

// Most tiles any wave owns inside one LDS chunk.
static int tiles_per_wave(int64_t n_kt, const SmallCfg& c)
{
    int64_t chunk_tiles = c.kc / TILE_K;
    if (chunk_tiles > n_kt) chunk_tiles = n_kt;
    return (int)((chunk_tiles + c.ks - 1) / c.ks);
}

template <typename Kern, typename Args>
static int launch_small(Kern kern, const char* what, const Args& a, const SmallCfg& c, size_t lds,
                        hipStream_t stream)
{
    if (int rc = ensure_dynamic_lds((const void*)kern, lds, what)) return rc;
    const dim3 grid((unsigned)((a.n_cb + c.cbw - 1) / c.cbw)), block(64 * c.cbw * c.ks);
    hipLaunchKernelGGL(kern, grid, block, lds, stream, a, c);
    return check_launch(what);
}


}  // namespace w2
