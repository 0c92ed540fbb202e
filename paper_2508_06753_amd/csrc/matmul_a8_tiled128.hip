// w2a8 for prefill, 128-row tiles: the compute-bound regime (Sec. III-C, GEMM
// results) on the int8 matrix cores.  Measured on MI355X, what limits this
// method there is vector-instruction issue: a SIMD issues one vector
// instruction, matrix ones included, about every four clocks, and per matrix
// instruction (16 clocks of matrix pipe) the method needs 256/G fmas to apply
// the group scales (Sec. II-D dequant, per group) plus 7/RI shift/mask
// instructions to up-convert (Sec. II-C), RI = row tiles that share a weight
// operand.  The 64-row kernel (RI = 4) runs at 5.2 vector instructions per
// matrix instruction; this one halves the up-convert share with 128-row wave
// tiles (RI = 8 x CJ = 2 column blocks of v_mfma_i32_16x16x64_i8) and spreads
// the remaining vector work evenly under the matrix instructions:
//   - workgroup 128 rows x 256 columns (eight waves of 128 x 32, one workgroup
//     per CU) or 128 x 128 (four waves, two per CU); a stage is 128 k = one
//     group of G = 128, 32 matrix instructions per wave;
//   - activations go through LDS (row stride 160 B: conflict-free operand
//     reads).  Three buffers: stage s reads buffers s and s+1 and writes the rows
//     of stage s+2, one barrier per stage.  Five buffers (eight-wave workgroups):
//     the pair of stages (2S, 2S+1) reads stages 2S .. 2S+2 and writes stages
//     2S+3 and 2S+4, five different buffers, one barrier per pair, so the waves
//     of a workgroup may be a stage apart inside a pair.  Rows are loaded from
//     global memory two stages before they go to LDS;
//   - the weights go from global memory to registers (the packed dword IS the
//     matrix operand), one 16-byte load per lane, column block and 256-k tile,
//     a tile ahead;
//   - every wave is software-pipelined on its own: under a stage's matrix
//     instructions it reads the second k-step's operands and the next stage's
//     first ones, up-converts one operand ahead, and dequantises a finished
//     column block in two halves (16 fmas per eight matrix instructions);
//   - dequant in ONE fma per accumulator: a group starts from BIAS = 2^21 (the
//     third MFMA operand), so acc = BIAS + 64*sum is positive and below 2^23 and
//     its bit pattern read as binary32 is the denormal acc * 2^-149:
//     y += as_float(acc) * (sw * 2^64); the bias term is taken out every 16
//     stages and at the end.  Requires fp32 denormals (the build keeps them and
//     the source refuses fast-math) and |sw| < 2^63.  (Starting from the bit
//     pattern of 1.5 * 2^23 instead, a normal number, is no faster -- denormal
//     operands cost the fma nothing here -- and carries six times the bias,
//     which costs the near-zero outputs their accuracy.)
#include <hip/hip_runtime.h>

#include <type_traits>

#include "w2_small_common.h"

#if defined(__HIP_DEVICE_COMPILE__) && defined(__FAST_MATH__)
#error "the one-fma dequant reads int32 accumulators as fp32 denormals: do not build with fast-math / flush-to-zero"
#endif

namespace w2 {

namespace t128 {

constexpr int RI = 8;                              // 16-row tiles per wave
constexpr int CJ = 2;                              // 16-column blocks per wave
constexpr int BM = 16 * RI, BK = 128;
constexpr int WN = 16 * CJ;
constexpr int A_STRIDE = BK + 32;                  // 32 mod 64 bytes: conflict-free A-operand reads
constexpr int A_BUF = BM * A_STRIDE;
// LDS buffers: 3 with a barrier after every stage; 5 with a barrier after every other stage (eight-wave
// workgroups, one per CU: the waves of a workgroup may then drift a stage apart inside a pair)
constexpr int nbuf_of(int bn) { return bn >= 256 ? 5 : 3; }
constexpr int E_STRIDE = WN * 2 + 16;              // epilogue: bytes per LDS row of a wave's result
constexpr int BIAS = 1 << 21;                      // > 64 * 127 * 2 * 128 = 2 080 768
constexpr float BIAS_F = 0x1p-128f;                // BIAS read as a float: 2^21 * 2^-149
constexpr int waves_of(int bn) { return bn / WN; }
constexpr int SX_BYTES = BM * 4;                   // the tile's activation scales, parked for the epilogue
constexpr int lds_bytes(int bn)
{
    return nbuf_of(bn) * A_BUF > waves_of(bn) * BM * E_STRIDE ? nbuf_of(bn) * A_BUF : waves_of(bn) * BM * E_STRIDE;
}

__device__ __forceinline__ v4i upconvert4(uint32_t w)
{
    v4i u;
    u[0] = (int)((w << 6) & 0xC0C0C0C0u);
    u[1] = (int)((w << 4) & 0xC0C0C0C0u);
    u[2] = (int)((w << 2) & 0xC0C0C0C0u);
    u[3] = (int)(w & 0xC0C0C0C0u);
    return u;
}

template <int G>
struct WTile {
    uint4 w[CJ];                                   // 16 bytes of codes per column block: dword t = k 64t .. 64t+63
    uint32_t s[CJ][G == 128 ? 1 : 2];              // the lane's column: 2 (G=128) or 4 (G=64) bf16 group scales
};

// SPLIT: K cut into gridDim.y near-equal ranges of whole 256-k tiles (c_lo tiles each, one more for the first
// c_rem ranges), one grid slice each; a range is entered by moving the base pointers, its fp32 results go to the
// workspace and a second launch sums them (Sec. II-D, K-splitting for the smaller shapes).  An instantiation of
// its own: the unsplit kernel is compiled exactly as before.
template <int G, bool DBG, int BN, bool SPLIT = false>
__global__ void __launch_bounds__(64 * waves_of(BN), BN >= 256 ? 1 : 2)
a8_tiled128_kernel(A8Args a, int tiles_m, int tiles_n, int group_m, int c_lo, int c_rem)
{
    constexpr int WAVES = waves_of(BN), THREADS = 64 * WAVES;
    constexpr int GPT = TILE_K / G;
    constexpr int CPT = THREADS / BM;              // threads per activation row: 4 or 2
    constexpr int NV = BK / CPT / 16;              // 16-byte pieces per thread and stage: 2 or 4
    constexpr bool TWO_SETS = NV <= 2;             // two register sets: a load has two stages to land
    constexpr int NBUF = nbuf_of(BN);
    constexpr int WR = NBUF == 3 ? 2 : 3;          // stage s writes the activations of stage s + WR
    static_assert(NBUF == 3 || TWO_SETS, "five buffers go with two register sets");
    extern __shared__ __align__(16) int8_t smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wn = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int q = lane >> 4, l16 = lane & 15;

    // workgroup -> tile: one contiguous chunk of ids per XCD (consecutive ids go to different XCDs),
    // bands of group_m row tiles inside, so that the workgroups resident on an XCD share activation rows
    // and weight columns through that XCD's L2
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

    const char* wb[CJ];
    const char* sb[CJ];
#pragma unroll
    for (int j = 0; j < CJ; ++j) {
        int64_t c = tile_n * (BN / TILE_N) + wn * CJ + j;
        c = c < a.n_cb ? c : a.n_cb - 1;                     // clamp: loads stay in bounds
        wb[j] = reinterpret_cast<const char*>(a.codes + c * a.n_kt * 256);
        sb[j] = reinterpret_cast<const char*>(a.scales + c * a.n_kt * TILE_N * GPT);
    }
    uint32_t w_lane = (uint32_t)lane * 16u;
    uint32_t s_lane = (uint32_t)l16 * (GPT * 2u);
    int64_t nkt = a.n_kt;                                    // tiles this workgroup multiplies
    int64_t kt0 = 0;                                         // the first of them
    if constexpr (SPLIT) {
        const int z = (int)blockIdx.y;
        kt0 = (int64_t)z * c_lo + min(z, c_rem);
        nkt = c_lo + (z < c_rem ? 1 : 0);
#pragma unroll
        for (int j = 0; j < CJ; ++j) {
            wb[j] += kt0 * 1024;
            sb[j] += kt0 * (TILE_N * GPT * 2);
        }
    }

    // global -> LDS copy: CPT threads per row, NV 16-byte pieces each; rows past M repeat the last row.
    // Lane offsets stay below 128 * K <= 2^31.
    const int cp_row = tid / CPT, cp_seg = tid % CPT;
    int64_t cp_m = m0 + cp_row;
    if (cp_m >= a.M) cp_m = a.M - 1;
    const char* cp_base = reinterpret_cast<const char*>(a.xq) + m0 * a.K + kt0 * TILE_K;  // uniform
    // piece v of a thread is the row's 16-byte piece v * CPT + cp_seg: the CPT threads of a row store CPT
    // consecutive pieces per instruction, so eight lanes (two or four rows) never share an LDS bank
    // (with NV consecutive pieces per thread a row's last piece fell on the next row's first bank)
    uint32_t cp_lane = (uint32_t)((cp_m - m0) * a.K) + (uint32_t)cp_seg * 16u;
    const int cp_dst = cp_row * A_STRIDE + cp_seg * 16;
    constexpr int CP_STEP = CPT * 16;              // bytes between a thread's pieces

    v4i acc[RI][CJ];
    float y[RI][CJ][4];
    float ssum[CJ] = {};                                     // sum of sw * 2^64 over the groups folded into y
    const v4i biasv = {BIAS, BIAS, BIAS, BIAS};
#pragma unroll
    for (int i = 0; i < RI; ++i)
#pragma unroll
        for (int j = 0; j < CJ; ++j) {
            acc[i][j] = biasv;
#pragma unroll
            for (int r = 0; r < 4; ++r) y[i][j][r] = 0.0f;
        }

    const int64_t n_st = nkt * 2;                            // stages of 128 k
    // plain named registers (arrays and structs of them ended up in scratch memory)
    uint4 p00, p01, p02 = make_uint4(0, 0, 0, 0), p03 = p02;         // set 0
    uint4 p10 = p02, p11 = p02;                                      // set 1 (eight-wave workgroups)
    auto load_a = [&](int64_t st, uint4& v0, uint4& v1, uint4& v2, uint4& v3) {
        st = min(st, n_st - 1);                              // past the end: re-read the last stage (never used)
        const char* p = cp_base + st * BK;                   // uniform
        asm volatile("" : "+v"(cp_lane));                    // keeps "scalar base + 32-bit offset" addressing
        v0 = *reinterpret_cast<const uint4*>(p + cp_lane);
        v1 = *reinterpret_cast<const uint4*>(p + cp_lane + CP_STEP);
        if constexpr (NV > 2) {
            v2 = *reinterpret_cast<const uint4*>(p + cp_lane + 2 * CP_STEP);
            v3 = *reinterpret_cast<const uint4*>(p + cp_lane + 3 * CP_STEP);
        }
    };
    auto store_a = [&](int buf, const uint4& v0, const uint4& v1, const uint4& v2, const uint4& v3) {
        int8_t* dst = smem + buf * A_BUF + cp_dst;
        *reinterpret_cast<uint4*>(dst) = v0;
        *reinterpret_cast<uint4*>(dst + CP_STEP) = v1;
        if constexpr (NV > 2) {
            *reinterpret_cast<uint4*>(dst + 2 * CP_STEP) = v2;
            *reinterpret_cast<uint4*>(dst + 3 * CP_STEP) = v3;
        }
    };
    auto load_w = [&](int64_t kt, WTile<G>& r) {
        kt = min(kt, nkt - 1);
        const int64_t w_off = kt * 1024;
        const int64_t s_off = kt * (TILE_N * GPT * 2);
        asm volatile("" : "+v"(w_lane), "+v"(s_lane));
#pragma unroll
        for (int j = 0; j < CJ; ++j) {
            r.w[j] = *reinterpret_cast<const uint4*>(wb[j] + w_off + w_lane);
            if constexpr (G == 128) {
                r.s[j][0] = *reinterpret_cast<const uint32_t*>(sb[j] + s_off + s_lane);
            } else {
                const uint2 v = *reinterpret_cast<const uint2*>(sb[j] + s_off + s_lane);
                r.s[j][0] = v.x;
                r.s[j][1] = v.y;
            }
        }
    };

    // the tile's activation scales, fetched now (unconditionally) and parked in LDS for the epilogue: loaded
    // there they would cost every workgroup a memory round trip with nothing to hide it
    float* sx_lds = reinterpret_cast<float*>(smem + lds_bytes(BN));
    const float sx_mine = DBG ? 0.f : a.sx[min(m0 + (tid & (BM - 1)), a.M - 1)];

    // prologue: stages 0 and 1 go to LDS; the registers then hold stage 2 (and 3)
    WTile<G> w0, w1;
    load_w(0, w0);
    {
        // every load of the prologue is issued before the first store waits: one memory round trip, not one
        // per stage (nothing else runs on the CU meanwhile: a workgroup has it to itself)
        const uint4 zero4 = make_uint4(0, 0, 0, 0);
        uint4 t0a, t0b, t0c = zero4, t0d = zero4, t1a, t1b, t1c = zero4, t1d = zero4, t2a = zero4, t2b = zero4, t2c = zero4, t2d = zero4;
        load_a(0, t0a, t0b, t0c, t0d);
        load_a(1, t1a, t1b, t1c, t1d);
        if constexpr (WR == 3) load_a(2, t2a, t2b, t2c, t2d);
        load_a(WR, p00, p01, p02, p03);
        if constexpr (TWO_SETS) load_a(WR + 1, p10, p11, p02, p03);
        store_a(0, t0a, t0b, t0c, t0d);
        store_a(1, t1a, t1b, t1c, t1d);
        if constexpr (WR == 3) store_a(2, t2a, t2b, t2c, t2d);
    }
    if (tid < BM) sx_lds[tid] = sx_mine;
    __syncthreads();

    const int8_t* a_base = smem + l16 * A_STRIDE + q * 16;

    // y += as_float(acc) * (sw * 2^64) for rows [i0, i0 + 4) of column block j
    auto dequant_half = [&](int j, int i0, float swS, int64_t g) {
#pragma unroll
        for (int i = i0; i < i0 + RI / 2; ++i) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if constexpr (DBG) {
                    const int64_t m = m0 + i * 16 + 4 * q + r;
                    const int64_t n = n0 + wn * WN + j * 16 + l16;
                    if (g >= 0 && m < a.M && n < a.N)
                        a.acc_out[(m * (a.K / G) + g) * a.N + n] = (acc[i][j][r] - BIAS) >> 6;
                }
                y[i][j][r] = fmaf(__int_as_float(acc[i][j][r]), swS, y[i][j][r]);
            }
        }
    };
    auto scale_of = [&](const WTile<G>& w, int j, int h, int t) -> float {
        // G = 128: the stage's group is group h of the tile; G = 64: k-step t of stage h is group 2h + t
        const uint32_t pair = G == 128 ? w.s[j][0] : w.s[j][h];
        const int hi = G == 128 ? h : t;
        return __uint_as_float(hi ? (pair & 0xffff0000u) : (pair << 16)) * 0x1p64f;
    };
    auto dword_of = [&](const WTile<G>& w, int j, int h, int t) -> uint32_t {
        const int d = 2 * h + t;
        return d == 0 ? w.w[j].x : d == 1 ? w.w[j].y : d == 2 ? w.w[j].z : w.w[j].w;
    };

    v4i a0[RI], a1[RI];
#pragma unroll
    for (int i = 0; i < RI; ++i) a0[i] = *reinterpret_cast<const v4i*>(a_base + i * 16 * A_STRIDE);
    v4i b_next = upconvert4(w0.w[0].x);                      // operand (k-step 0, column block 0) of the coming stage
    float pend_sw = 0.f;                                     // column block 1 of the previous stage: nothing yet
    int64_t pend_g = -1;
    int buf = 0;

    // One stage (G = 128: one group).  Order of the matrix instructions: column block 0, k-steps 0 and 1
    // (blocks A, B), then column block 1 (blocks C, D).  Vector work under them:
    //   A: second k-step's operands from LDS, up-convert (1,0), dequant the previous stage's column 1, rows 0..63
    //   B: up-convert (0,1), dequant the previous stage's column 1, rows 64..127
    //   C: up-convert (1,1), dequant this stage's column 0, rows 0..63
    //   D: next stage's first operands from LDS, up-convert its (0,0), dequant column 0, rows 64..127
    auto stage = [&](int64_t it, auto hc, const WTile<G>& wc, WTile<G>& wnx) {
        constexpr int h = decltype(hc)::value;
        const int buf1 = buf == NBUF - 1 ? 0 : buf + 1;
        const int bufw = buf + WR >= NBUF ? buf + WR - NBUF : buf + WR;
        if constexpr (TWO_SETS && h == 1) {                  // activations of stage it+2
            store_a(bufw, p10, p11, p02, p03);
            load_a(it + WR + 2, p10, p11, p02, p03);
        } else {
            store_a(bufw, p00, p01, p02, p03);
            load_a(it + WR + (TWO_SETS ? 2 : 1), p00, p01, p02, p03);
        }
        if constexpr (h == 0) load_w((it >> 1) + 1, wnx);
        __builtin_amdgcn_sched_barrier(0);                   // all loads are issued up here, unconditionally
        const int8_t* ab = a_base + buf * A_BUF;
        const int8_t* abn = a_base + buf1 * A_BUF;
        const WTile<G>& wn_tile = h == 1 ? wnx : wc;         // where the next stage finds its weights
        static_assert(G == 128, "this schedule is written for one group per stage");
        const float sw0 = scale_of(wc, 0, h, 0), sw1 = scale_of(wc, 1, h, 0);
        const int64_t g = it;                                // group index = stage index (G = 128)

        const v4i b00 = b_next;
        // Each block is a scheduling region of its own (sched_barrier at its end): the vector work placed in a
        // block reads only accumulators finished at least one block (eight matrix instructions) earlier.  In one
        // region the scheduler pulled the fmas up to right behind the matrix instruction that produces their
        // operand, and every such pair stalls the wave until the matrix pipe has written the result (measured:
        // 2070 TOP/s; 4290 with the same fmas reading other registers).
        auto interleave = [&](bool with_lds) {               // per matrix instruction: [one LDS read] three vector instructions
#pragma unroll
            for (int k = 0; k < RI; ++k) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                if (with_lds) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        };
        // block A
#pragma unroll
        for (int i = 0; i < RI; ++i) a1[i] = *reinterpret_cast<const v4i*>(ab + i * 16 * A_STRIDE + 64);
        const v4i b10 = upconvert4(dword_of(wc, 0, h, 1));
#pragma unroll
        for (int i = 0; i < RI; ++i) acc[i][0] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a0[i], b00, biasv, 0, 0, 0);
        dequant_half(1, 0, pend_sw, pend_g);
        interleave(true);
        // block B
        const v4i b01 = upconvert4(dword_of(wc, 1, h, 0));
#pragma unroll
        for (int i = 0; i < RI; ++i) acc[i][0] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a1[i], b10, acc[i][0], 0, 0, 0);
        dequant_half(1, RI / 2, pend_sw, pend_g);
        ssum[1] += pend_sw;
        interleave(false);
        // block C
        const v4i b11 = upconvert4(dword_of(wc, 1, h, 1));
#pragma unroll
        for (int i = 0; i < RI; ++i) acc[i][1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a0[i], b01, biasv, 0, 0, 0);
        dequant_half(0, 0, sw0, g);
        interleave(false);
        // block D
#pragma unroll
        for (int i = 0; i < RI; ++i) a0[i] = *reinterpret_cast<const v4i*>(abn + i * 16 * A_STRIDE);
        b_next = upconvert4(dword_of(wn_tile, 0, h ^ 1, 0));
#pragma unroll
        for (int i = 0; i < RI; ++i) acc[i][1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a1[i], b11, acc[i][1], 0, 0, 0);
        dequant_half(0, RI / 2, sw0, g);
        ssum[0] += sw0;
        pend_sw = DBG ? 1.0f : sw1;
        pend_g = g;
        interleave(true);
        buf = buf1;
        if constexpr (NBUF == 3 || h == 1) __syncthreads();
    };

    // one 256-k tile (two stages) per iteration; the next tile's weights arrive in w1 meanwhile and move
    // to w0 at the end (every load and every register write is unconditional: registers written under a
    // condition end up in scratch memory)
    for (int64_t kt = 0; kt < nkt; ++kt) {
        stage(kt * 2, std::integral_constant<int, 0>{}, w0, w1);
        stage(kt * 2 + 1, std::integral_constant<int, 1>{}, w0, w1);
        w0 = w1;
        if ((kt & 7) == 7) {
            // take the accumulated bias term out every 16 stages, so that the running sums never carry
            // more than 16 stages of it (the rounding error stays near 2^-14 of the result, whatever K is)
#pragma unroll
            for (int j = 0; j < CJ; ++j) {
                // column 1 of the stage just finished is still pending: its scale is not in ssum[1] yet
                const float corr = ssum[j] * BIAS_F;
                ssum[j] = 0.f;
#pragma unroll
                for (int i = 0; i < RI; ++i)
#pragma unroll
                    for (int r = 0; r < 4; ++r) y[i][j][r] -= corr;
            }
        }
    }
    // the very last stage's column block 1
    dequant_half(1, 0, pend_sw, pend_g);
    dequant_half(1, RI / 2, pend_sw, pend_g);
    ssum[1] += pend_sw;
    if constexpr (DBG) return;

    // y_true = (y - BIAS*2^-149 * ssum) * 2^(149-64) * 2^-6 * sx.  The wave's 128 x 32 result goes through
    // LDS (its own region; the barrier at the end of the last stage freed the activation buffers) and
    // leaves as 16-byte stores.
    int8_t* ebase = smem + wn * (BM * E_STRIDE);
    uint16_t* eb = reinterpret_cast<uint16_t*>(ebase);
    const bool gated = a.epi.act == ACT_SILU_MUL;
    float bias[CJ];
#pragma unroll
    for (int j = 0; j < CJ; ++j) {
        const int64_t n = n0 + wn * WN + j * 16 + l16;
        bias[j] = (a.epi.bias && n < a.N) ? bf16_to_f32(a.epi.bias[n]) : 0.f;
    }
    // (one copy of the loop per epilogue, picked here: a choice per element would have the compiler
    // evaluate the SiLU for every output and select afterwards)
    float cj[CJ];
#pragma unroll
    for (int j = 0; j < CJ; ++j) cj[j] = ssum[j] * BIAS_F;
    if constexpr (SPLIT) {
        // this range's results, dequantised, as fp32 rows of the workspace: the wave's 128 x 32 tile goes
        // through LDS 64 rows at a time (rows padded by 16 bytes: conflict-free both ways; the wave reads
        // back only what it wrote) and leaves as 16-byte stores in 128-byte runs
        constexpr int P_STRIDE = WN * 4 + 16;
        static_assert(waves_of(BN) * 64 * P_STRIDE <= lds_bytes(BN), "partial-result staging fits the activation buffers");
        float* dst = a.part + (int64_t)blockIdx.y * a.M * a.N;
        int8_t* pbase = smem + wn * (64 * P_STRIDE);
        const int prow = lane >> 3, pcol = (lane & 7) * 4;   // eight lanes per row piece
        const int64_t n = n0 + wn * WN + pcol;
#pragma unroll
        for (int h = 0; h < RI / 4; ++h) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float4 s4 = *reinterpret_cast<const float4*>(sx_lds + (h * 4 + i) * 16 + 4 * q);
                const float sr[4] = {s4.x, s4.y, s4.z, s4.w};
#pragma unroll
                for (int r = 0; r < 4; ++r)
#pragma unroll
                    for (int j = 0; j < CJ; ++j)
                        *reinterpret_cast<float*>(pbase + (i * 16 + 4 * q + r) * P_STRIDE + (j * 16 + l16) * 4) =
                            (y[h * 4 + i][j][r] - cj[j]) * (sr[r] * 0x1p79f);
            }
#pragma unroll
            for (int p = 0; p < 8; ++p) {
                const int row = p * 8 + prow;
                const int64_t m = m0 + h * 64 + row;
                const float4 v = *reinterpret_cast<const float4*>(pbase + row * P_STRIDE + pcol * 4);
                if (m < a.M && n < a.N) *reinterpret_cast<float4*>(dst + m * a.N + n) = v;   // N % 8 == 0: all 4 or none
            }
        }
        return;
    }
    auto emit = [&](auto mode_c) {
        constexpr int MODE = decltype(mode_c)::value;        // ACT_NONE, ACT_SILU, ACT_SILU_MUL
#pragma unroll
        for (int i = 0; i < RI; ++i) {
            const float4 s4 = *reinterpret_cast<const float4*>(sx_lds + i * 16 + 4 * q);     // rows 4q .. 4q+3 of row tile i
            const float sr[4] = {s4.x, s4.y, s4.z, s4.w};
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = i * 16 + 4 * q + r;
                const float t = sr[r] * 0x1p79f;
                float z[CJ];
#pragma unroll
                for (int j = 0; j < CJ; ++j) z[j] = (y[i][j][r] - cj[j]) * t + bias[j];
                if constexpr (MODE == ACT_SILU_MUL) {
                    eb[row * (E_STRIDE / 2) + l16] = f32_to_bf16_rne(silu_f32(z[0]) * z[1]);
                } else {
                    static_assert(CJ == 2, "one packed conversion per row");
                    const uint32_t pk = MODE == ACT_SILU ? pack_bf16x2(silu_f32(z[0]), silu_f32(z[1])) : pack_bf16x2(z[0], z[1]);
                    eb[row * (E_STRIDE / 2) + l16] = (uint16_t)pk;
                    eb[row * (E_STRIDE / 2) + 16 + l16] = (uint16_t)(pk >> 16);
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

template <bool DBG, int BN, bool SPLIT = false>
static int launch(const A8Args& a, int splits, hipStream_t stream)
{
    constexpr int WAVES = waves_of(BN);
    const int tiles_m = (int)((a.M + BM - 1) / BM);
    const int tiles_n = (int)((a.N + BN - 1) / BN);
    // Row tiles per band: the 32 workgroups resident on an XCD cover group_m row tiles x 32 / group_m column
    // tiles and fetch group_m MiB of activations and 16 / group_m MiB of weights per round at K = 8192: 4
    // moves the least through the XCD's L2 (measured as fast as 8 at M = 2048, 2 % faster at M = 4096).
    const int group_m = a.tune.tiled_group_m ? a.tune.tiled_group_m : 4;
    constexpr int lds = lds_bytes(BN) + SX_BYTES;
    auto kern = a8_tiled128_kernel<128, DBG, BN, SPLIT>;
    if (int rc = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), lds, "w2_matmul_a8[tiled 128]")) return rc;
    const dim3 grid((unsigned)((int64_t)tiles_m * tiles_n), (unsigned)(SPLIT ? splits : 1)), block(64 * WAVES);
    hipLaunchKernelGGL(kern, grid, block, lds, stream, a, tiles_m, tiles_n, group_m, (int)(a.n_kt / (SPLIT ? splits : 1)),
                       (int)(a.n_kt % (SPLIT ? splits : 1)));
    int rc = check_launch("w2_matmul_a8[tiled 128]");
    if (rc || !SPLIT) return rc;
    return launch_splitk_reduce(a.part, splits, a.M, a.N, a.Y, a.ldy, a.epi, stream);
}

}  // namespace t128

// G = 128 only (a stage is one group).
bool a8_tiled128_supports(const A8Args& a) { return a.G == 128; }

// K ranges across workgroups for the 128-row kernel: with room for partial results, 256-column workgroups
// (one per CU) times floor(256 / tiles) ranges -- one round, never more -- up to 8, at least two 256-k tiles
// each, at most 64 MiB of partial results (the rule that came out of the w2a16 kernel's sweeps, which has
// the same tiling).
int a8_tiled128_splits(int64_t M, int64_t N, int64_t n_kt, int64_t cap, const w2_tuning_t& tune)
{
    if (tune.splitk > 0) return (int)max((int64_t)1, min((int64_t)tune.splitk, min(cap, n_kt)));
    const int64_t t256 = ((M + 127) / 128) * ((N + 255) / 256);
    int64_t s = 256 / max(t256, (int64_t)1);
    s = min(s, (int64_t)8);
    s = min(s, n_kt / 2);
    s = min(s, ((int64_t)64 << 20) / (M * N * (int64_t)sizeof(float)));
    s = min(s, cap);
    return s < 2 ? 1 : (int)s;
}

// splits: K ranges across workgroups (1 = none); the caller decides (a8_tiled128_splits is the rule).
int launch_a8_tiled128(const A8Args& a, int splits, hipStream_t stream)
{
    const int64_t wgs256 = ((a.M + 127) / 128) * ((a.N + 255) / 256);
    const int64_t cap = a.part ? (int64_t)(a.part_bytes / ((size_t)a.M * a.N * sizeof(float))) : 0;
    if (a.acc_out || splits > cap || splits > a.n_kt) splits = 1;
    if (splits >= 2) {
        if (a.tune.tiled_bn == 128) return t128::launch<false, 128, true>(a, splits, stream);
        return t128::launch<false, 256, true>(a, splits, stream);
    }
    const int bn = a.tune.tiled_bn == 128 || a.tune.tiled_bn == 256 ? a.tune.tiled_bn : wgs256 <= 128 ? 128 : 256;
    if (a.acc_out) return bn == 128 ? t128::launch<true, 128>(a, 1, stream) : t128::launch<true, 256>(a, 1, stream);
    return bn == 128 ? t128::launch<false, 128>(a, 1, stream) : t128::launch<false, 256>(a, 1, stream);
}

}  // namespace w2
