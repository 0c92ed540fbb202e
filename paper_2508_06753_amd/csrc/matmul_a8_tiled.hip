// w2a8 for large M (prefill): the compute-bound regime (Sec. III-C, GEMM
// results) on the int8 matrix cores.  The workgroup / wave tile hierarchy
// plays the role of the wg_tile / sg_tile split of Sec. II-D, re-derived for
// CDNA4: a 128(M) x 256(N) workgroup tile, eight waves of 64 x 64, each wave
// 4 x 4 tiles of v_mfma_i32_16x16x64_i8.
//   - activations (int8) are staged through LDS, double-buffered, 256 k per
//     stage, rows padded by 16 B so ds_read_b128 is conflict-free;
//   - the 2-bit weights never touch LDS: the packed layout IS the MFMA
//     B-operand layout, so each lane loads its dwords straight from global
//     memory and up-converts them in registers (Sec. II-C "up-convert and
//     compute"), reused across the wave's four row tiles;
//   - the dequant (Sec. II-D: int32 -> float, x scale) is applied per group of
//     G k's in registers: y += sw * float(acc); the activation scale and the
//     exact 1/64 of the up-convert are applied once in the epilogue.
#include <hip/hip_runtime.h>

#include "w2_internal.h"

namespace w2 {

typedef int v4i __attribute__((ext_vector_type(4)));

namespace tiled {

constexpr int BM = 128, BN = 256, BK = TILE_K;
constexpr int THREADS = 512;
constexpr int A_STRIDE = BK + 16;                 // bytes per LDS row
constexpr int A_BUF = BM * A_STRIDE;              // bytes per stage
constexpr int WM = 64, WN = 64;                   // wave tile

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ v4i upconvert(uint32_t w)
{
    v4i u;
    u[0] = (int)((w << 6) & 0xC0C0C0C0u);
    u[1] = (int)((w << 4) & 0xC0C0C0C0u);
    u[2] = (int)((w << 2) & 0xC0C0C0C0u);
    u[3] = (int)(w & 0xC0C0C0C0u);
    return u;
}

struct WRegs {
    uint4 w[4];         // four column blocks of this wave, one k tile
    uint32_t s[4][2];   // their group scales (bf16 pairs)
};

template <int G>
__device__ __forceinline__ void load_w(const A8Args& a, const int64_t (&cb)[4], int64_t kt, int lane,
                                       WRegs& r)
{
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int64_t tile = cb[j] * a.n_kt + kt;
        r.w[j] = *reinterpret_cast<const uint4*>(a.codes + (tile * 64 + lane) * 4);
        if constexpr (G == 128) {
            r.s[j][0] = *reinterpret_cast<const uint32_t*>(a.scales + (tile * TILE_N + (lane & 15)) * 2);
            r.s[j][1] = 0;
        } else {
            const uint2 s = *reinterpret_cast<const uint2*>(a.scales + (tile * TILE_N + (lane & 15)) * 4);
            r.s[j][0] = s.x; r.s[j][1] = s.y;
        }
    }
}

template <int G>
__device__ __forceinline__ float w_scale(const WRegs& r, int j, int gi)
{
    const uint32_t pair = (G == 128 || gi < 2) ? r.s[j][0] : r.s[j][1];
    return (gi & 1) ? __uint_as_float(pair & 0xffff0000u) : __uint_as_float(pair << 16);
}

template <int G, bool DBG>
__global__ void __launch_bounds__(THREADS)
a8_tiled_kernel(A8Args a, int tiles_m, int tiles_n, int group_m)
{
    extern __shared__ __align__(16) int8_t smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 2, wn = wave & 3;
    const int q = lane >> 4, l16 = lane & 15;

    // Workgroup -> tile.  Consecutive workgroup ids go to different XCDs (round
    // robin over 8), so ids are first regrouped into 8 contiguous chunks, one
    // per XCD, and inside a chunk walked in bands of group_m row tiles so that
    // the workgroups resident on an XCD share activation rows and weight
    // columns through that XCD's L2.
    const int64_t total = (int64_t)tiles_m * tiles_n;
    int64_t id = blockIdx.x;
    {
        const int64_t per_xcd = (total + 7) / 8;
        const int64_t x = id & 7, i = id >> 3;
        const int64_t rid = x * per_xcd + i;
        // chunks are equal-sized only if total % 8 == 0; otherwise keep ids as they are
        if (total % 8 == 0) id = rid;
    }
    const int64_t band = id / ((int64_t)group_m * tiles_n);
    const int64_t first_m = band * group_m;
    const int gm = (int)min((int64_t)group_m, tiles_m - first_m);
    const int64_t in_band = id - band * group_m * tiles_n;
    const int64_t tile_m = first_m + in_band % gm;
    const int64_t tile_n = in_band / gm;

    const int64_t m0 = tile_m * BM, n0 = tile_n * BN;
    int64_t cb[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int64_t c = tile_n * (BN / TILE_N) + wn * 4 + j;
        cb[j] = c < a.n_cb ? c : a.n_cb - 1;                 // clamp: loads stay in bounds
    }

    // global -> LDS copy assignment: 16 threads per 256-byte row, 32 rows per pass
    const int cp_v = tid & 15, cp_r = tid >> 4;
    const int8_t* cp_src[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        int64_t m = m0 + cp_r + 32 * p;
        if (m >= a.M) m = a.M - 1;                           // padded rows repeat the last row
        cp_src[p] = a.xq + m * a.K + cp_v * 16;
    }
    const int cp_dst = cp_r * A_STRIDE + cp_v * 16;

    v4i acc[4][4];
    float y[4][4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            acc[i][j] = (v4i){0, 0, 0, 0};
#pragma unroll
            for (int r = 0; r < 4; ++r) y[i][j][r] = 0.0f;
        }

    // prologue: stage 0
    uint4 areg[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) areg[p] = *reinterpret_cast<const uint4*>(cp_src[p]);
    WRegs wcur;
    load_w<G>(a, cb, 0, lane, wcur);
#pragma unroll
    for (int p = 0; p < 4; ++p)
        *reinterpret_cast<uint4*>(smem + cp_dst + 32 * p * A_STRIDE) = areg[p];
    __syncthreads();

    const int8_t* a_base = smem + (wm * WM + l16) * A_STRIDE + q * 16;
    constexpr int GPT = TILE_K / G;

    for (int64_t kt = 0; kt < a.n_kt; ++kt) {
        const int buf = (int)(kt & 1);
        const bool more = kt + 1 < a.n_kt;
        if (more) {
#pragma unroll
            for (int p = 0; p < 4; ++p)
                areg[p] = *reinterpret_cast<const uint4*>(cp_src[p] + (kt + 1) * BK);
        }
        const int8_t* ab = a_base + buf * A_BUF;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            v4i aop[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                aop[i] = *reinterpret_cast<const v4i*>(ab + i * 16 * A_STRIDE + t * 64);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t wd = t == 0 ? wcur.w[j].x : t == 1 ? wcur.w[j].y
                                  : t == 2 ? wcur.w[j].z : wcur.w[j].w;
                const v4i bop = upconvert(wd);
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(aop[i], bop, acc[i][j], 0, 0, 0);
            }
            if (G == 64 || (t & 1)) {
                const int gi = G == 64 ? t : t >> 1;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float sw = w_scale<G>(wcur, j, gi);
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            if constexpr (DBG) {
                                const int64_t m = m0 + wm * WM + i * 16 + 4 * q + r;
                                const int64_t n = n0 + wn * WN + j * 16 + l16;
                                if (m < a.M && n < a.N)
                                    a.acc_out[(m * (a.K / G) + kt * GPT + gi) * a.N + n] = acc[i][j][r] >> 6;
                            }
                            y[i][j][r] = fmaf(sw, (float)acc[i][j][r], y[i][j][r]);
                        }
                        acc[i][j] = (v4i){0, 0, 0, 0};
                    }
                }
            }
        }
        if (more) {
            int8_t* dst = smem + (buf ^ 1) * A_BUF + cp_dst;
#pragma unroll
            for (int p = 0; p < 4; ++p)
                *reinterpret_cast<uint4*>(dst + 32 * p * A_STRIDE) = areg[p];
            load_w<G>(a, cb, kt + 1, lane, wcur);
        }
        __syncthreads();
    }
    if constexpr (DBG) return;

#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int64_t m = m0 + wm * WM + i * 16 + 4 * q + r;
            if (m >= a.M) continue;
            const float s = a.sx[m] * 0.015625f;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int64_t n = n0 + wn * WN + j * 16 + l16;
                if (n < a.N) a.Y[m * a.ldy + n] = f32_to_bf16_rne(y[i][j][r] * s);
            }
        }
    }
}

}  // namespace tiled

int launch_a8_tiled(const A8Args& a, hipStream_t stream)
{
    using namespace tiled;
    const int tiles_m = (int)((a.M + BM - 1) / BM);
    const int tiles_n = (int)((a.N + BN - 1) / BN);
    const size_t lds = 2 * A_BUF;
    int group_m = env_int("W2_TILED_GROUP_M", 4);
    if (group_m < 1) group_m = 1;
    const dim3 grid((unsigned)((int64_t)tiles_m * tiles_n)), block(THREADS);
    hipError_t e = hipSuccess;
    if (a.G == 128) {
        if (a.acc_out) {
            e = hipFuncSetAttribute((const void*)a8_tiled_kernel<128, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e == hipSuccess) hipLaunchKernelGGL((a8_tiled_kernel<128, true>), grid, block, lds, stream, a, tiles_m, tiles_n, group_m);
        } else {
            e = hipFuncSetAttribute((const void*)a8_tiled_kernel<128, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e == hipSuccess) hipLaunchKernelGGL((a8_tiled_kernel<128, false>), grid, block, lds, stream, a, tiles_m, tiles_n, group_m);
        }
    } else {
        if (a.acc_out) {
            e = hipFuncSetAttribute((const void*)a8_tiled_kernel<64, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e == hipSuccess) hipLaunchKernelGGL((a8_tiled_kernel<64, true>), grid, block, lds, stream, a, tiles_m, tiles_n, group_m);
        } else {
            e = hipFuncSetAttribute((const void*)a8_tiled_kernel<64, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e == hipSuccess) hipLaunchKernelGGL((a8_tiled_kernel<64, false>), grid, block, lds, stream, a, tiles_m, tiles_n, group_m);
        }
    }
    if (e != hipSuccess) {
        set_error("w2_matmul_a8[tiled]: hipFuncSetAttribute: %s", hipGetErrorString(e));
        return -5;
    }
    return check_launch("w2_matmul_a8[tiled]");
}

}  // namespace w2
