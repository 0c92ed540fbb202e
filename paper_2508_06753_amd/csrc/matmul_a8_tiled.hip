// w2a8 for large M (prefill): the compute-bound regime (Sec. III-C, GEMM
// results) on the int8 matrix cores.  The workgroup / wave tile hierarchy
// plays the role of the wg_tile / sg_tile split of Sec. II-D, re-derived for
// CDNA4: a 64(M) x 256(N) workgroup tile, eight waves of 64 x 32 (RI = 4 row
// tiles x CJ = 2 column blocks of v_mfma_i32_16x16x64_i8; two workgroups per
// CU, four waves per SIMD).  Measured on MI355X: the chip is power-limited in
// this kernel (its speed depends on how many operand bits toggle), so what
// counts is work per result: vector instructions per matrix instruction (the
// SIMD issues one vector instruction, matrix ones included, every four clocks
// or so) and bytes moved.
//   - activations (int8) are staged through LDS, three buffers, 128 k per
//     stage, rows padded by 32 B;
//   - the 2-bit weights never touch LDS: the packed layout IS the MFMA
//     B-operand layout, so each lane loads its dwords (64 bits per column
//     block and stage) straight from global memory and up-converts them in
//     registers (Sec. II-C "up-convert and compute"), reused across the wave's
//     four row tiles; addresses are scalar base + 32-bit lane offset;
//   - all loads are issued unconditionally (clamped past the end) at the top of
//     a stage and pinned there: with loads under a condition the compiler
//     cannot count how many are in flight, and its waits for the previous
//     stage's registers then also wait for the loads just issued;
//   - the dequant (Sec. II-D: int32 -> float, x scale) runs once per group of G
//     k's on the accumulators of a wave, in ONE fma per accumulator: every
//     group starts from the constant BIAS = 2^21 (a third MFMA operand, never
//     written), so the int32 result acc = BIAS + 64*sum is positive and below
//     2^23, i.e. its bit pattern read as binary32 is the denormal
//     acc * 2^-149; y += as_float(acc) * (sw * 2^64) needs no int->float
//     conversion.  The bias term, BIAS * 2^-149 * sum_g sw_g * 2^64, is
//     subtracted every 8 stages and in the epilogue; while it rides along it
//     exceeds the wanted sum by about 2^9, which leaves 15 of fp32's 24 bits
//     for a bf16 result.  The int32 group accumulators themselves stay exact
//     (acc - BIAS is what the debug export stores).  A column block is
//     dequantised under the matrix instructions of the next one;
//   - results leave through LDS as 16-byte stores.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "w2_internal.h"

#if defined(__HIP_DEVICE_COMPILE__) && defined(__FAST_MATH__)
#error "the one-fma dequant reads int32 accumulators as fp32 denormals: do not build with fast-math / flush-to-zero"
#endif

namespace w2 {

typedef int v4i __attribute__((ext_vector_type(4)));

namespace tiled {

constexpr int RI = 4;                             // 16-row tiles per wave
constexpr int CJ = 2;                             // 16-column blocks per wave
constexpr int BM = 16 * RI, BK = 128;                 // BK: k per pipeline stage (half a packed tile)
// BN (columns per workgroup, template parameter): 256 = eight waves, or 128 = four waves when the
// problem would otherwise yield too few workgroups to fill the chip
constexpr int waves_of(int bn) { return bn / (16 * CJ); }
// bytes per LDS row: with a stride of 32 mod 64 bytes the A-operand reads (row = lane & 15, 16-byte
// piece = lane >> 4) run at full LDS rate; measured, a 16-byte pad costs 1.75x on those reads
constexpr int A_STRIDE = BK + 32;
constexpr int A_BUF = BM * A_STRIDE;              // bytes per stage
constexpr int WM = BM, WN = 16 * CJ;                // wave tile
constexpr int E_STRIDE = WN * 2 + 16;             // epilogue: bytes per LDS row of a wave's result
constexpr int P_STRIDE = WN * 4 + 16;             // split-K: bytes per LDS row of a wave's fp32 partial result
// LDS layout after the main loop: [epilogue regions | partial results of the groups 1..KW-1 | fp32 staging]
constexpr int exch_off(int waves) { return waves * BM * E_STRIDE; }
constexpr int pstage_off(int waves, int kw) { return kw > 1 ? exch_off(waves) + (kw - 1) * waves * BM * WN * 4 : 0; }
constexpr int wgs_per_cu(int threads, int wd = 2)
{
    // a weight window deeper than two stages needs more than 128 registers: two waves per SIMD
    if (wd > 2) return threads > 256 ? 1 : 2;
    return threads > 512 ? 1 : threads <= 256 && RI * CJ <= 8 ? 4 : ((RI * CJ <= 16 && threads <= 256) || (RI * CJ <= 8) ? 2 : 1);
}
constexpr int BIAS = 1 << 21;                     // > 64 * 127 * 2 * 128 = 2 080 768

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

// Weights and scales of one stage (128 k) for the wave's column blocks.
struct WStage {
    uint2 w[CJ];      // two dwords = two 64-k steps
    uint32_t s[CJ];   // G=128: one bf16 scale (low half); G=64: two bf16 scales
};

// wb[j] / sb[j]: wave-uniform byte pointers to column block j's codes / scales (scalar registers);
// w_lane / s_lane: this lane's byte offset inside a packed tile.  The stage offset is uniform, so
// every load is "scalar base + 32-bit lane offset" and costs no vector address arithmetic.
template <int G>
__device__ __forceinline__ void load_w(const char* const (&wb)[CJ], const char* const (&sb)[CJ],
                                       uint32_t w_lane, uint32_t s_lane, int64_t it, WStage& r)
{
    const int64_t kt = it >> 1;
    const int h = (int)(it & 1);
    const int64_t w_off = (kt * 256 + h * 2) * 4;
    const int64_t s_off = G == 128 ? (kt * (TILE_N * 2) + h) * 2 : (kt * (TILE_N * 4) + h * 2) * 2;
#pragma unroll
    for (int j = 0; j < CJ; ++j) {
        r.w[j] = *reinterpret_cast<const uint2*>(wb[j] + w_off + w_lane);
        if constexpr (G == 128)
            r.s[j] = *reinterpret_cast<const uint16_t*>(sb[j] + s_off + s_lane);
        else
            r.s[j] = *reinterpret_cast<const uint32_t*>(sb[j] + s_off + s_lane);
    }
}

// KW > 1: K-splitting inside the workgroup (Sec. II-D) for problems with too few output tiles to give
// every SIMD a wave: KW groups of waves_of(BN) waves each run this kernel on their own K range (the
// group index extends the split coordinate; the host guarantees equal ranges, so every group meets
// the same barriers) with activation buffers of their own; the partial results meet in LDS, group 0
// adds them in a fixed order and stores.
//
// WD: weight stages in flight per wave (the one being multiplied included).  Two are enough when the
// weights come out of L2 (many row tiles share them); a problem of one or two row tiles streams them
// from HBM once, and a stage's arithmetic is far shorter than a memory round trip: there every wave
// keeps WD - 1 = 7 stages (7 KiB) on their way.
template <int G, bool DBG, int BN, int KW, int WD>
__global__ void __launch_bounds__(64 * waves_of(BN) * KW, wgs_per_cu(64 * waves_of(BN) * KW, WD))
a8_tiled_kernel(A8Args a, int tiles_m, int tiles_n, int group_m, int splits)
{
    constexpr int WAVES = waves_of(BN), THREADS = 64 * WAVES;      // per group
    (void)WAVES;
    extern __shared__ __align__(16) int8_t smem_all[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int grp = KW > 1 ? wave / WAVES : 0;
    const int tid = (int)threadIdx.x - grp * THREADS;              // thread index inside the group
    int8_t* const smem = smem_all + grp * (3 * A_BUF);             // this group's activation buffers
    const int wm = 0, wn = KW > 1 ? wave % WAVES : wave;
    const int q = lane >> 4, l16 = lane & 15;

    // Workgroup -> tile.  Consecutive workgroup ids go to different XCDs (round
    // robin over 8), so ids are first regrouped into 8 contiguous chunks, one
    // per XCD, and inside a chunk walked in bands of group_m row tiles so that
    // the workgroups resident on an XCD share activation rows and weight
    // columns through that XCD's L2.
    const int64_t total = (int64_t)tiles_m * tiles_n;
    int64_t id = blockIdx.x;
    if (total % 8 == 0) id = (id & 7) * (total >> 3) + (id >> 3);
    const int64_t band = id / ((int64_t)group_m * tiles_n);
    const int64_t first_m = band * group_m;
    const int gm = (int)min((int64_t)group_m, tiles_m - first_m);
    const int64_t in_band = id - band * group_m * tiles_n;
    const int64_t tile_m = first_m + in_band % gm;
    const int64_t tile_n = in_band / gm;
    const int64_t m0 = tile_m * BM, n0 = tile_n * BN;

    // per column block: wave-uniform base pointers of its codes and scales
    const char* wb[CJ];
    const char* sb[CJ];
#pragma unroll
    for (int j = 0; j < CJ; ++j) {
        int64_t c = tile_n * (BN / TILE_N) + wn * CJ + j;
        c = c < a.n_cb ? c : a.n_cb - 1;                     // clamp: loads stay in bounds
        wb[j] = reinterpret_cast<const char*>(a.codes + c * a.n_kt * 256);
        sb[j] = reinterpret_cast<const char*>(a.scales + c * a.n_kt * TILE_N * (TILE_K / G));
    }
    uint32_t w_lane = (uint32_t)lane * 16u;
    uint32_t s_lane = (uint32_t)l16 * (uint32_t)(TILE_K / G) * 2u;

    // global -> LDS copy: CPT threads per 128-byte row piece, CPB bytes (NV 16-byte pieces) each.  Rows past
    // M repeat the last row; the lane offset (< 64 K) fits 32 bits.
    constexpr int CPT = THREADS / BM, CPB = BK / CPT;        // threads per row, bytes each: 2 x 64, 4 x 32 or 8 x 16
    constexpr int NV = CPB / 16;
    static_assert(CPB == 64 || CPB == 32 || CPB == 16, "copy geometry");
    const int cp_row = tid / CPT, cp_seg = tid % CPT;
    int64_t cp_m = m0 + cp_row;
    if (cp_m >= a.M) cp_m = a.M - 1;
    const char* cp_base = reinterpret_cast<const char*>(a.xq) + m0 * a.K;          // uniform
    uint32_t cp_lane = (uint32_t)((cp_m - m0) * a.K) + (uint32_t)cp_seg * CPB;
    const int cp_dst = cp_row * A_STRIDE + cp_seg * CPB;

    v4i acc[RI][CJ];
    float y[RI][CJ][4];
    float ssum[CJ] = {};                   // sum of the scaled group scales per column block
    const v4i biasv = {BIAS, BIAS, BIAS, BIAS};
#pragma unroll
    for (int i = 0; i < RI; ++i)
#pragma unroll
        for (int j = 0; j < CJ; ++j) {
            acc[i][j] = biasv;
#pragma unroll
            for (int r = 0; r < 4; ++r) y[i][j][r] = 0.0f;
        }

    // Pipeline: the activations of stage it+1 sit in registers during stage it-1 and are written
    // to LDS at the top of stage it (three LDS buffers); the weights of stage it+1 are loaded at
    // the top of stage it into the other of two register sets.  Every global load has a whole
    // stage to land before anything waits for it.
    // this workgroup's K range (split-K: blockIdx.y of `splits` near-equal ranges of whole 256-k tiles)
    const int64_t sy = (int64_t)blockIdx.y * KW + grp, ns = (int64_t)splits * KW;
    const int64_t it_b = a.n_kt * sy / ns * 2;
    const int64_t n_it = a.n_kt * (sy + 1) / ns * 2;               // stages [it_b, n_it): an even number, >= 2
    // The empty asm statements keep the zero-extension of a lane offset next to its load, which is
    // what lets the compiler pick the "scalar base + 32-bit vector offset" addressing mode.
    // (pieces passed one by one: with the array handed over as a whole the compiler kept it in scratch memory)
    auto load_a4 = [&](int64_t it, uint4& r0, uint4& r1, uint4& r2, uint4& r3) {
        const char* p = cp_base + it * BK;                   // uniform
        asm volatile("" : "+v"(cp_lane));
        r0 = *reinterpret_cast<const uint4*>(p + cp_lane);
        if constexpr (NV > 1) r1 = *reinterpret_cast<const uint4*>(p + cp_lane + 16);
        if constexpr (NV > 2) {
            r2 = *reinterpret_cast<const uint4*>(p + cp_lane + 32);
            r3 = *reinterpret_cast<const uint4*>(p + cp_lane + 48);
        }
    };
    auto store_a4 = [&](int8_t* dst, const uint4& r0, const uint4& r1, const uint4& r2, const uint4& r3) {
        *reinterpret_cast<uint4*>(dst) = r0;
        if constexpr (NV > 1) *reinterpret_cast<uint4*>(dst + 16) = r1;
        if constexpr (NV > 2) {
            *reinterpret_cast<uint4*>(dst + 32) = r2;
            *reinterpret_cast<uint4*>(dst + 48) = r3;
        }
    };
#define W2_PIECES(x) x[0], x[NV > 1 ? 1 : 0], x[NV > 2 ? 2 : 0], x[NV > 2 ? 3 : 0]
    // Vector memory loads complete in order, so a wait for an activation load also waits for every weight
    // load issued before it: with a deep weight window the activations need the same lead, or each
    // stage would still wait for the weights of the stage before.  AQ register sets hold them on
    // their way (stage s in set (s - it_b) % AQ); LEAD = stages between a load and its LDS store + 1.
    constexpr int AQ = WD > 2 ? WD : 1, LEAD = WD > 2 ? WD : 2;
    uint4 aq[AQ][NV];
#pragma unroll
    for (int i = 0; i < AQ; ++i)
#pragma unroll
        for (int v = 1; v < NV; ++v) aq[i][v] = make_uint4(0, 0, 0, 0);   // (dead stores that keep the array in registers)
    WStage wq[WD];
    load_a4(it_b, W2_PIECES(aq[0]));
#pragma unroll
    for (int i = 0; i < WD - 1; ++i) {
        load_w<G>(wb, sb, w_lane, s_lane, min(it_b + i, n_it - 1), wq[i]);
        if constexpr (WD > 2) load_a4(min(it_b + i + 1, n_it - 1), W2_PIECES(aq[(i + 1) % AQ]));
    }
    if constexpr (WD > 2) __builtin_amdgcn_sched_barrier(0);
    store_a4(smem + cp_dst, W2_PIECES(aq[0]));               // (waits for the oldest load only)
    if constexpr (WD == 2) load_a4(it_b + 1, W2_PIECES(aq[0]));
    __syncthreads();

    const int8_t* a_base = smem + (wm * WM + l16) * A_STRIDE + q * 16;

    // y += as_float(acc) * (sw * 2^64) for one column block, then restart the group
    auto dequant_col = [&](int j, float swS, int64_t g) {
#pragma unroll
        for (int i = 0; i < RI; ++i) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if constexpr (DBG) {
                    const int64_t m = m0 + wm * WM + i * 16 + 4 * q + r;
                    const int64_t n = n0 + wn * WN + j * 16 + l16;
                    if (m < a.M && n < a.N)
                        a.acc_out[(m * (a.K / G) + g) * a.N + n] = (acc[i][j][r] - BIAS) >> 6;
                }
                y[i][j][r] = fmaf(__int_as_float(acc[i][j][r]), swS, y[i][j][r]);
            }
        }
        ssum[j] += swS;
    };
    // The last column block of a group is dequantised under the first matrix instructions of the
    // NEXT group (its accumulators are not written again before that group reaches the last
    // column), so no stage ends with vector work that has nothing to hide under.
    float pend_sw = 0.f;                                     // nothing pending yet: adds BIAS * 0
    int64_t pend_g = 0;

    // One stage: wc holds this stage's weights, wnx (the set the stage before has just used up)
    // receives those of stage it + WD - 1.
    auto stage = [&](int64_t it, int buf, int buf_next, const WStage& wc, WStage& wnx, uint4 (&ast)[NV], uint4 (&ald)[NV]) {
        // No branch around the loads: past the end they re-read the last stage (and the last
        // LDS write lands in a buffer nobody reads any more).  With loads under a condition the
        // compiler cannot count how many are in flight and its waits for the previous stage's
        // registers also wait for the loads just issued, i.e. a full memory round trip per stage.
        {
            store_a4(smem + buf_next * A_BUF + cp_dst, W2_PIECES(ast));  // activations of stage it+1
            asm volatile("" : "+v"(w_lane), "+v"(s_lane));
            load_w<G>(wb, sb, w_lane, s_lane, min(it + (WD - 1), n_it - 1), wnx);
        }
        load_a4(min(it + LEAD, n_it - 1), W2_PIECES(ald));
        // keep the loads up here: the scheduler otherwise sinks them to their first use, one stage on
        __builtin_amdgcn_sched_barrier(0);
        const int8_t* ab = a_base + buf * A_BUF;
        float swS[CJ][2];
#pragma unroll
        for (int j = 0; j < CJ; ++j) {
            if constexpr (G == 128) {
                swS[j][0] = __uint_as_float(wc.s[j] << 16) * 0x1p64f;
                swS[j][1] = 0.f;
            } else {
                swS[j][0] = __uint_as_float(wc.s[j] << 16) * 0x1p64f;
                swS[j][1] = __uint_as_float(wc.s[j] & 0xffff0000u) * 0x1p64f;
            }
        }
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            v4i aop[RI];
#pragma unroll
            for (int i = 0; i < RI; ++i)
                aop[i] = *reinterpret_cast<const v4i*>(ab + i * 16 * A_STRIDE + t * 64);
            const bool first = (G == 64) || t == 0;          // first k-step of a group starts from BIAS
            const bool last = (G == 64) || t == 1;
#pragma unroll
            for (int j = 0; j < CJ; ++j) {
                const v4i bop = upconvert(t == 0 ? wc.w[j].x : wc.w[j].y);
#pragma unroll
                for (int i = 0; i < RI; ++i)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(aop[i], bop, first ? biasv : acc[i][j], 0, 0, 0);
                // the previous column's results are ready by now: dequantise them under these MFMAs
                if (last && j > 0) dequant_col(j - 1, swS[j - 1][G == 64 ? t : 0], it * (128 / G) + (G == 64 ? t : 0));
                if (CJ > 1 && first && j == 0) {
                    if constexpr (DBG) { if (pend_sw != 0.f) dequant_col(CJ - 1, pend_sw, pend_g); }
                    else dequant_col(CJ - 1, pend_sw, pend_g);
                }
            }
            if (last) {
                if constexpr (CJ > 1) {
                    pend_sw = DBG ? 1.0f : swS[CJ - 1][G == 64 ? t : 0];
                    pend_g = it * (128 / G) + (G == 64 ? t : 0);
                } else {                                     // a single column block has nothing to hide under
                    dequant_col(0, swS[0][G == 64 ? t : 0], it * (128 / G) + (G == 64 ? t : 0));
                }
            }
        }
    };

    // take the accumulated bias term out every 8 stages, so that the running sums never carry more
    // than 8 stages of it (keeps the rounding error near 2^-15 of the result, whatever K is)
    auto settle = [&]() {
#pragma unroll
        for (int j = 0; j < CJ; ++j) {
            const float corr = ssum[j] * 0x1p-128f;         // BIAS * 2^-149 = 2^-128
            ssum[j] = 0.f;
#pragma unroll
            for (int i = 0; i < RI; ++i)
#pragma unroll
                for (int r = 0; r < 4; ++r) y[i][j][r] -= corr;
        }
    };
    int buf = 0;
    for (int64_t it = it_b; it < n_it; it += WD) {
#pragma unroll
        for (int i = 0; i < WD; i += 2) {
            if constexpr (WD > 2) {
                if (i > 0 && it + i >= n_it) break;          // (stages come in pairs; uniform over the workgroup)
            }
            const int b1 = buf == 2 ? 0 : buf + 1;
            const int b2 = b1 == 2 ? 0 : b1 + 1;
            stage(it + i, buf, b1, wq[i], wq[(i + WD - 1) % WD], aq[(i + 1) % AQ], aq[(i + LEAD) % AQ]);
            __syncthreads();
            stage(it + i + 1, b1, b2, wq[i + 1], wq[i], aq[(i + 2) % AQ], aq[(i + 1 + LEAD) % AQ]);
            buf = b2;
            if (((it + i) & 7) == 6) settle();
            __syncthreads();
        }
    }
    if constexpr (CJ > 1) dequant_col(CJ - 1, pend_sw, pend_g);   // the very last group's last column
    if constexpr (DBG) return;
    if constexpr (KW > 1) {
        // the groups' partial results (bias term taken out) meet in LDS, behind the epilogue's regions;
        // element e of a wave's 64 x 32 tile sits at [e][lane]: conflict-free both ways
        float* pr = reinterpret_cast<float*>(smem_all + exch_off(WAVES)) + (int64_t)wn * (RI * 4 * CJ * 64) + lane;
#pragma unroll
        for (int i = 0; i < RI; ++i)
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int j = 0; j < CJ; ++j) {
                    y[i][j][r] -= ssum[j] * 0x1p-128f;
                    if (grp > 0) pr[((grp - 1) * WAVES * (RI * 4 * CJ) + (i * 4 + r) * CJ + j) * 64] = y[i][j][r];
                }
#pragma unroll
        for (int j = 0; j < CJ; ++j) ssum[j] = 0.f;
        __syncthreads();
        if (grp > 0) return;
        for (int g = 0; g < KW - 1; ++g)
#pragma unroll
            for (int i = 0; i < RI; ++i)
#pragma unroll
                for (int r = 0; r < 4; ++r)
#pragma unroll
                    for (int j = 0; j < CJ; ++j) y[i][j][r] += pr[(g * WAVES * (RI * 4 * CJ) + (i * 4 + r) * CJ + j) * 64];
    }

    // y_true = (y - BIAS*2^-149 * ssum) * 2^(149-64) * 2^-6 * sx   (2^-128 = BIAS * 2^-149)
    // Each lane holds single columns of four rows per tile, which would make 2-byte stores in
    // 32-byte runs; the wave's 64 x 64 result goes through LDS instead (its own
    // region; the barrier at the end of the last stage freed the activation buffers) and leaves
    // as 16-byte stores, eight lanes per 128-byte row piece.
    if (a.part) {
        // split-K: this range's results, dequantised, go to the workspace as fp32 rows.  A lane holds single
        // columns of four rows per tile (4-byte stores in 64-byte runs: measured, 5 us of a 29 us launch on
        // 28672 x 8192 at M = 64); the wave's 64 x 32 tile goes through LDS (a region of its own, rows padded
        // by 16 bytes: conflict-free both ways) and leaves as 16-byte stores in 128-byte runs.
        float* dst = a.part + (int64_t)blockIdx.y * a.M * a.N;
        int8_t* pbase = smem_all + pstage_off(WAVES, KW) + wn * (BM * P_STRIDE);
        const int prow = lane >> 3, pcol = (lane & 7) * 4;   // eight lanes per row piece
        float sxr[BM / 8];
#pragma unroll
        for (int p = 0; p < BM / 8; ++p) {
            const int64_t m = m0 + p * 8 + prow;
            sxr[p] = a.sx[m < a.M ? m : a.M - 1];
        }
#pragma unroll
        for (int i = 0; i < RI; ++i)
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int j = 0; j < CJ; ++j)
                    *reinterpret_cast<float*>(pbase + (i * 16 + 4 * q + r) * P_STRIDE + (j * 16 + l16) * 4) =
                        (y[i][j][r] - ssum[j] * 0x1p-128f) * 0x1p79f;
        // the wave reads back only what it wrote itself: LDS operations of one wave complete in order
        const int64_t n = n0 + wn * WN + pcol;
#pragma unroll
        for (int p = 0; p < BM / 8; ++p) {
            const int row = p * 8 + prow;
            const int64_t m = m0 + row;
            float4 v = *reinterpret_cast<const float4*>(pbase + row * P_STRIDE + pcol * 4);
            v.x *= sxr[p]; v.y *= sxr[p]; v.z *= sxr[p]; v.w *= sxr[p];
            if (m < a.M && n < a.N) *reinterpret_cast<float4*>(dst + m * a.N + n) = v;   // N % 8 == 0: all 4 or none
        }
        return;
    }
    int8_t* ebase = smem_all + wn * (BM * E_STRIDE);
    uint16_t* eb = reinterpret_cast<uint16_t*>(ebase);
    // fused epilogue (Sec. II-D: bias and activation applied while the outputs are in registers).
    // The gated form combines the wave's two column blocks, an even (gate) and an odd (up) one,
    // into one block of outputs.
    const bool gated = a.epi.act == ACT_SILU_MUL;
    float bias[CJ];
#pragma unroll
    for (int j = 0; j < CJ; ++j) {
        const int64_t n = n0 + wn * WN + j * 16 + l16;
        bias[j] = (a.epi.bias && n < a.N) ? __uint_as_float((uint32_t)a.epi.bias[n] << 16) : 0.f;
    }
    // (one copy of the loop per epilogue, picked here: a choice per element would have the compiler
    // evaluate the SiLU for every output and select afterwards)
    auto emit = [&](auto mode_c) {
        constexpr int MODE = decltype(mode_c)::value;        // ACT_NONE, ACT_SILU, ACT_SILU_MUL
#pragma unroll
        for (int i = 0; i < RI; ++i) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = i * 16 + 4 * q + r;
                const int64_t m = m0 + row;
                const float s = a.sx[m < a.M ? m : a.M - 1];
                float z[CJ];
#pragma unroll
                for (int j = 0; j < CJ; ++j) z[j] = (y[i][j][r] - ssum[j] * 0x1p-128f) * 0x1p79f * s + bias[j];
                if constexpr (CJ == 2 && MODE == ACT_SILU_MUL) {
                    eb[row * (E_STRIDE / 2) + l16] = f32_to_bf16_rne(z[0] / (1.0f + __expf(-z[0])) * z[1]);
                } else {
#pragma unroll
                    for (int j = 0; j < CJ; ++j) {
                        const float v = MODE == ACT_SILU ? z[j] / (1.0f + __expf(-z[j])) : z[j];
                        eb[row * (E_STRIDE / 2) + j * 16 + l16] = f32_to_bf16_rne(v);
                    }
                }
            }
        }
    };
    if (gated) emit(std::integral_constant<int, ACT_SILU_MUL>{});
    else if (a.epi.act == ACT_SILU) emit(std::integral_constant<int, ACT_SILU>{});
    else emit(std::integral_constant<int, ACT_NONE>{});
    // the wave reads back only what it wrote itself: LDS operations of one wave complete in order
    const int wcols = gated ? WN / 2 : WN;                   // output columns of this wave
    const int lpr = wcols * 2 / 16;                          // lanes per row piece (16 bytes each): 4 or 2
    const int rpp = 64 / lpr;                                // rows per pass
    const int64_t ncol = (gated ? (n0 + wn * WN) / 2 : n0 + wn * WN) + (lane % lpr) * 8;   // first of this lane's 8 columns
    const int64_t n_out = gated ? a.N / 2 : a.N;
    for (int p = 0; p < BM / rpp; ++p) {
        const int row = p * rpp + lane / lpr;
        const int64_t m = m0 + row;
        const uint4 v = *reinterpret_cast<const uint4*>(ebase + row * E_STRIDE + (lane % lpr) * 16);
        if (m < a.M && ncol < n_out) *reinterpret_cast<uint4*>(a.Y + m * a.ldy + ncol) = v;   // N % 8 == 0: all 8 or none
    }
}

#undef W2_PIECES

}  // namespace tiled

template <int G, bool DBG, int BN, int KW = 1, int WD = 2>
static int launch_tiled(const A8Args& a_in, int splits, hipStream_t stream)
{
    using namespace tiled;
    constexpr int WAVES = waves_of(BN), THREADS = 64 * WAVES * KW;
    A8Args a = a_in;
    if (splits < 2 || DBG) { a.part = nullptr; splits = 1; }
    const int tiles_m = (int)((a.M + BM - 1) / BM);
    const int tiles_n = (int)((a.N + BN - 1) / BN);
    // three activation stages per group; the epilogue regions (and behind them the groups' partial results) reuse them
    const size_t act = (size_t)KW * 3 * A_BUF;
    const size_t epi = (size_t)WAVES * BM * E_STRIDE + (size_t)(KW - 1) * WAVES * BM * WN * sizeof(float);
    const size_t pst = a.part ? (size_t)pstage_off(WAVES, KW) + (size_t)WAVES * BM * P_STRIDE : 0;
    const size_t lds = max(max(act, epi), pst);
    const int group_m = a.tune.tiled_group_m ? a.tune.tiled_group_m : 8;
    const dim3 grid((unsigned)((int64_t)tiles_m * tiles_n), (unsigned)splits), block(THREADS);
    auto kern = a8_tiled_kernel<G, DBG, BN, KW, WD>;
    if (int rc = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), lds, "w2_matmul_a8[tiled]")) return rc;
    hipLaunchKernelGGL(kern, grid, block, lds, stream, a, tiles_m, tiles_n, group_m, splits);
    int rc = check_launch("w2_matmul_a8[tiled]");
    if (rc || !a.part) return rc;
    return launch_splitk_reduce(a.part, splits, a.M, a.N, a.Y, a.ldy, a.epi, stream);
}

// 256 columns per workgroup unless that leaves the chip's 512 workgroup slots clearly underfilled
static int tiled_bn(int64_t M, int64_t N, const w2_tuning_t& tune)
{
    const int64_t wgs256 = ((M + tiled::BM - 1) / tiled::BM) * ((N + 255) / 256);
    int bn = tune.tiled_bn;
    if (bn != 64 && bn != 128 && bn != 256) bn = wgs256 < 400 ? 128 : 256;
    return bn;
}

// How a problem's K is cut: `splits` ranges across workgroups (partial results in the workspace, summed
// by a second launch) times `kw` ranges inside a workgroup (128-column workgroups only).
struct TiledPlan { int bn, splits, kw; };

static TiledPlan tiled_plan(int64_t M, int64_t N, int64_t n_kt, int64_t cap, const w2_tuning_t& tune)
{
    TiledPlan p;
    p.bn = tiled_bn(M, N, tune);
    const int64_t tiles_m = (M + tiled::BM - 1) / tiled::BM;
    const int forced_s = tune.splitk;                        // tuning and tests: 1 = never, n = n parts if they fit
    if (p.bn == 256) {
        // many output tiles: split only to fill the chip (splitk_plan)
        const int64_t wgs_n = tiles_m * ((N + 255) / 256);
        if (forced_s > 0) p.splits = (int)min((int64_t)forced_s, min(max(cap, (int64_t)1), n_kt));
        else p.splits = splitk_plan(wgs_n, n_kt, tune.splitk_min_tiles ? tune.splitk_min_tiles : 12, M, N, cap);
        p.kw = 1;
        return p;
    }
    // Fewer than 400 tiles of 64 x 256: from a few dozen to a few hundred workgroups against 256 CUs, so K is
    // cut both ways.  Every (splits, kw) that divides the tiles evenly is priced with a model fitted to sweeps
    // over 28672 x 8192, 14336 x 4096, 17408 x 5120, 4096 x 28672, 8192 x 8192, 4096 x 4096, 4096 x 6144,
    // 5120 x 7168 and 2048 x 2048 at M = 32..768:
    //   loop  = the work of the busiest CU at 1600 TOP/s: it gets ceil(workgroups / 256) workgroups (a CU holds
    //           one of 16 waves, two of 8, four of 4 at a time; more run in rounds, +10 %); with fewer than 8
    //           waves on the CU it runs at 0.55 of that rate (measured: 8 and 16 waves per CU run a stage in the
    //           same time); fewer workgroups than CUs cost another 15 % (the busy CUs queue more stages each);
    //   parts = 6 us for the second launch and both kernels' ends + the partial results written and read once
    //           at 3 TB/s.
    // 64-column workgroups (two waves per group, four groups) are priced too where they still fit the chip in
    // one round and K is not split across workgroups, at 30 % more per unit of work (every workgroup stages
    // the whole 64-row panel of activations for half the columns; fitted: 13.4 / 20.8 / 54.2 us at 6.3 / 10.7 /
    // 37.6 us of work): 4096 x 6144 at M = 65..128 13.1 against 15.5 us, 8192 x 8192 19.3 against 21.4, 4096 x
    // 4096 at M = 256 13.3 against 15.7.  In more than one round, or with K split on top, they lost everywhere
    // (14336 x 4096 at M = 384: 62 against 38 us).
    const double work_us = 2.0 * (double)(tiles_m * tiled::BM) * (double)N * (double)(n_kt * TILE_K) / 1600e6;
    const int64_t room = max(cap, (int64_t)1);
    int64_t s_lo = 1, s_hi = min(min((int64_t)16, room), max((int64_t)1, ((int64_t)16 << 20) / (M * N * (int64_t)sizeof(float))));
    if (forced_s > 0) s_lo = s_hi = min((int64_t)forced_s, min(room, n_kt));
    const int forced_kw = tune.tiled_kw;
    double best = 1e30;
    p.splits = (int)s_lo;
    p.kw = 1;
    auto price = [&](int bn, int kw, int64_t sp) {
        const int64_t wgs = tiles_m * ((N + bn - 1) / bn) * sp;
        const int64_t per_cu = (wgs + 255) / 256;                        // workgroups on the busiest CU
        const int64_t at_once = min(per_cu, (int64_t)(kw == 4 ? 1 : kw == 2 ? 2 : 4));
        const double waves = (double)(at_once * (bn / 32) * kw);
        const double rate = waves >= 8.0 ? 1.0 : 0.55;
        double loop = (double)per_cu * work_us * 256.0 / (double)wgs / rate;
        if (wgs < 256) loop /= 0.85;
        if (per_cu > at_once) loop *= 1.1;
        if (bn == 64) loop *= 1.3;
        const double parts = sp > 1 ? 6.0 + 2.0 * (double)sp * (double)M * (double)N * 4.0 / 3e6 : 0.0;
        return loop + parts;
    };
    bool found = false;
    for (int kw = 4; kw >= 1; kw >>= 1) {
        if (forced_kw && kw > forced_kw) continue;           // (a forced kw that does not divide the tiles falls back to the next smaller)
        for (int64_t sp = s_lo; sp <= s_hi && sp <= n_kt; ++sp) {
            if (kw > 1 && n_kt % (kw * sp) != 0) continue;
            if (forced_s <= 0 && sp > 1 && n_kt / (sp * kw) < 2) continue;
            const double t = price(p.bn, kw, sp);
            found = true;
            if (t < best) { best = t; p.splits = (int)sp; p.kw = kw; }
        }
        if (forced_kw && found) break;
    }
    // (an unsplit launch carries about 4 us of first loads and epilogue that the split launches' 6 us include;
    // the narrow workgroups one more; and they must win by 10 %: the model is that good and no better)
    if (tune.tiled_bn == 0 && forced_s <= 1 && (forced_kw == 0 || forced_kw == 4) && n_kt % 4 == 0 &&
        tiles_m * ((N + 63) / 64) <= 256 && price(64, 4, 1) + 5.0 < 0.9 * (best + (p.splits > 1 ? 0.0 : 4.0))) {
        p.bn = 64;
        p.splits = 1;
        p.kw = 4;
    }
    return p;
}

// Deep K with room for partial results: the 128-row kernel with its own K ranges (half the up-convert work per
// matrix instruction) instead of 64-row tiles.  Measured against the priced 64-row plan: 28672 x 8192 at
// M = 128 / 256 / 512 / 768 44 / 70 / 125 / 193 against 48 / 80 / 145 / 215 us, 17408 x 5120 at M = 256 / 512 / 768
// 36 / 56 / 77 against 40 / 77 / 88; at K = 14336 and below the 64-row plan holds its own (14336 x 4096 at
// M = 256: 27.5 against 29.4), and so it does below 256 rows at K = 17408.
static int deep128_splits(int64_t M, int64_t N, int64_t n_kt, int64_t G, int64_t cap, const w2_tuning_t& tune)
{
    if (tune.tiled_bm || G != 128 || !((n_kt >= 100 && M >= 128) || (n_kt >= 64 && M >= 256))) return 1;
    const int s = a8_tiled128_splits(M, N, n_kt, cap, tune);
    const int64_t t256 = ((M + 127) / 128) * ((N + 255) / 256);
    return s >= 2 && t256 * s >= 192 ? s : 1;
}

size_t a8_tiled_splitk_bytes(int64_t M, int64_t N, int64_t n_kt, int G, const w2_tuning_t& tune)
{
    const int s = max(tiled_plan(M, N, n_kt, 16, tune).splits, deep128_splits(M, N, n_kt, G, 16, tune));
    return s < 2 ? 0 : (size_t)s * M * N * sizeof(float);
}

template <int G, bool DBG>
static int launch_tiled_bn(const A8Args& a, hipStream_t stream)
{
    const int64_t cap = a.part ? (int64_t)(a.part_bytes / ((size_t)a.M * a.N * sizeof(float))) : 0;
    TiledPlan p = tiled_plan(a.M, a.N, a.n_kt, cap, a.tune);
    if (DBG) { p.splits = 1; p.kw = 1; }
    const int splits = p.splits;
    if constexpr (!DBG) {
        if (a.tune.tiled_wd == 8) {
            if (p.bn == 256) return launch_tiled<G, DBG, 256, 1, 8>(a, splits, stream);
            if (p.kw >= 2) return launch_tiled<G, DBG, 128, 2, 8>(a, splits, stream);
            return launch_tiled<G, DBG, 128, 1, 8>(a, splits, stream);
        }
        if (p.bn == 128 && p.kw == 4) return launch_tiled<G, DBG, 128, 4>(a, splits, stream);
        if (p.bn == 128 && p.kw == 2) return launch_tiled<G, DBG, 128, 2>(a, splits, stream);
        if (p.bn == 64 && p.kw == 4) return launch_tiled<G, DBG, 64, 4>(a, splits, stream);
        if (p.bn == 64 && p.kw == 2) return launch_tiled<G, DBG, 64, 2>(a, splits, stream);
    }
    if (p.bn == 64) return launch_tiled<G, DBG, 64>(a, splits, stream);
    return p.bn == 128 ? launch_tiled<G, DBG, 128>(a, splits, stream) : launch_tiled<G, DBG, 256>(a, splits, stream);
}

int launch_a8_tiled(const A8Args& a, hipStream_t stream)
{
    // 128-row tiles (half the up-convert work per matrix instruction) where the problem has the rows for
    // them and K is not split across workgroups
    {
        const int64_t cap = a.part ? (int64_t)(a.part_bytes / ((size_t)a.M * a.N * sizeof(float))) : 0;
        const int splits = a.acc_out ? 1 : tiled_plan(a.M, a.N, a.n_kt, cap, a.tune).splits;
        // 128-row tiles run one workgroup per CU, so a last round of workgroups that fills less than half the
        // chip costs a whole round (64-row workgroups share a CU in pairs and speed up when alone); with 224
        // tiles and more and a last round at least half full they win from M = 128 on (8192 x 57344 at M = 128:
        // 71 against 84 us; 4096 x 28672 at M = 384, 1.3 rounds: 66 against 57)
        const int64_t t128 = (a.M + 127) / 128 * ((a.N + 255) / 256);
        const bool fill_ok = t128 >= 768 || t128 % 256 == 0 || t128 % 256 >= 128;
        const bool want128 = a.tune.tiled_bm ? a.tune.tiled_bm == 128
                                             : a.M >= 1024 || (a.M >= 128 && t128 >= 224 && fill_ok);
        const int s_deep = a.acc_out ? 1 : deep128_splits(a.M, a.N, a.n_kt, a.G, cap, a.tune);
        if (a8_tiled128_supports(a)) {
            // forced 128-row tiles: that kernel's own rule for K ranges (or the forced count)
            if (a.tune.tiled_bm == 128) return launch_a8_tiled128(a, a8_tiled128_splits(a.M, a.N, a.n_kt, cap, a.tune), stream);
            if (s_deep >= 2) return launch_a8_tiled128(a, s_deep, stream);
            if (want128 && splits < 2) return launch_a8_tiled128(a, 1, stream);
        }
    }
    if (a.G == 128)
        return a.acc_out ? launch_tiled_bn<128, true>(a, stream) : launch_tiled_bn<128, false>(a, stream);
    return a.acc_out ? launch_tiled_bn<64, true>(a, stream) : launch_tiled_bn<64, false>(a, stream);
}

}  // namespace w2
