// w2a8 for medium M (9..64): between the memory-bound GEMV regime and the
// compute-bound GEMM regime of Sec. III-C.  The weight stream is still read
// exactly once ("up-convert and compute", Sec. II-C): a wave owns one 16-column
// block and every KS-th 256-k tile of it, up-converts each dword once and feeds
// it to RT row tiles of v_mfma_i32_16x16x64_i8 (M <= 16*RT), so the shift/mask
// cost per matrix instruction falls with M.  K is split across the waves of a
// workgroup (Sec. II-D, K-splitting for small shapes) and reduced through LDS in
// a fixed order; the dequant epilogue is fused (Sec. II-D).
//
// Schedule.  Eight waves: CBW = 2*TPC column blocks x KS = 4/TPC k-splits.  The
// activations go through LDS in chunks of 1024 k (four tiles; every wave works
// on TPC of them), one buffer: the next chunk is fetched into registers while
// the current one is being multiplied, and stored between two barriers.  The
// weight tiles run through a rolling window of eight per wave (8 KiB in
// flight): the load of tile s+8 is issued as soon as tile s has been consumed,
// whatever the chunk boundaries do.
#include <hip/hip_runtime.h>

#include "w2_small_common.h"

#if defined(__HIP_DEVICE_COMPILE__) && defined(__FAST_MATH__)
#error "the one-fma dequant reads int32 accumulators as fp32 denormals: do not build with fast-math / flush-to-zero"
#endif

namespace w2 {

// (column blocks per workgroup, K ranges) for a problem with room for `cap` fp32 copies of the output
MidmPlan midm_plan(int64_t M, int64_t n_cb, int64_t n_kt, int64_t cap, const w2_tuning_t& tune)
{
    constexpr int ROWS_PER_BAND = 64, CHUNK_TILES = 4;
    const int64_t bands = (M + ROWS_PER_BAND - 1) / ROWS_PER_BAND;
    const int64_t n_chunks = (n_kt + CHUNK_TILES - 1) / CHUNK_TILES;
    const int forced_cbw = tune.midm_cbw == 2 || tune.midm_cbw == 4 || tune.midm_cbw == 8 ? tune.midm_cbw : 0;
    MidmPlan p;
    // Deep K (14 chunks and more) and room for partial results: about 64 workgroups across the columns,
    // each as wide as that allows (every workgroup reads all M rows of its K range of the activations:
    // fewer, wider workgroups move less through L2), times enough K ranges for one workgroup per CU.
    // Measured at M = 64: 28672 x 8192 34 us against 57 us unsplit, 14336 x 4096 17 against 22 us; at
    // 8 chunks and fewer the partial results and the second launch cost more than they save.
    int64_t s = 1;
    p.cbw = forced_cbw;
    if (tune.splitk != 1 && cap >= 2 && (tune.splitk > 1 || n_chunks >= 14)) {
        if (!p.cbw) p.cbw = n_cb >= 8 * 64 ? 8 : n_cb >= 4 * 64 ? 4 : 2;
        const int64_t wgs = (n_cb + p.cbw - 1) / p.cbw * bands;
        s = tune.splitk > 1 ? tune.splitk : (256 + wgs / 2) / wgs;
        if (tune.splitk == 0) s = min(s, n_chunks / 3);
        s = min(min(s, n_chunks), min((int64_t)16, cap));
    }
    if (s < 2) {
        // K in one piece: as many column blocks per workgroup as still leave about one workgroup per CU
        s = 1;
        p.cbw = forced_cbw ? forced_cbw : n_cb >= 8 * 224 ? 8 : n_cb >= 4 * 224 ? 4 : 2;
    }
    p.splits = (int)s;
    return p;
}

namespace midm {

constexpr int THREADS = 512;
constexpr int CHUNK_TILES = 4;                               // k tiles per LDS chunk
constexpr int ROW_STRIDE = CHUNK_TILES * TILE_K + XS_PAD;    // bytes per LDS activation row
constexpr int D = 8;                                         // weight tiles in flight per wave
constexpr int ROWS_PER_BAND = 64;                            // rows one workgroup multiplies (RT <= 4 row tiles)

template <int G, int RT, int TPC, bool DBG, bool SPLIT>
__global__ void __launch_bounds__(THREADS)
a8_midm_kernel(A8Args a_all, int c_lo, int c_rem)
{
    // More than 64 rows: blockIdx.y picks a band of 64 rows; the bands stream the same weights (the
    // second one mostly out of L2), which pays when one band's workgroups would leave CUs idle.
    A8Args a = a_all;
    {
        const int64_t m_off = (int64_t)blockIdx.y * ROWS_PER_BAND;
        a.M = min((int64_t)ROWS_PER_BAND, a_all.M - m_off);
        a.xq += m_off * a.K;
        if (a.sx) a.sx += m_off;
        if (a.Y) a.Y += m_off * a.ldy;
        if (a.acc_out) a.acc_out += m_off * (a.K / G) * a.N;
        if (a.part) a.part += ((int64_t)blockIdx.z * a_all.M + m_off) * a.N;
    }
    constexpr int KS = CHUNK_TILES / TPC;                    // k-splits
    constexpr int CBW = 8 / KS;                              // column blocks per workgroup
    constexpr int NS = 2 * RT;                               // 16-byte activation pieces per thread and chunk
    constexpr int GPT = TILE_K / G;
    extern __shared__ __align__(16) int8_t smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int cbi = wave % CBW, ks = wave / CBW;
    const int q = lane >> 4, l16 = lane & 15;
    const int64_t cb = (int64_t)blockIdx.x * CBW + cbi;
    const bool cb_ok = cb < a.n_cb;
    const int64_t cbc = cb_ok ? cb : a.n_cb - 1;             // clamp: keeps loads in bounds
    const int64_t n = cb * TILE_N + l16;
    const int rows = (int)a.M;                               // 1..16*RT
    const int64_t row_stride = a.K;                          // bytes between activation rows in memory
    // Split-K across workgroups (Sec. II-D): blockIdx.z picks one of the near-equal ranges of whole 1024-k
    // chunks (c_lo chunks each, one more for the first c_rem ranges: no division here, ahead of the first
    // loads), and the workgroup stages only that K range of the activation rows.  The range is entered by
    // moving the base pointers: from here on the kernel sees a problem of n_kt tiles that starts at tile 0,
    // and the loop the compiler builds is the unsplit kernel's (around a run-time first chunk it was 5 %
    // slower on every shape).
    const int64_t kt_stride = a.n_kt;                        // tiles per column block in memory
    int64_t kt0 = 0;                                         // first tile of this workgroup's range
    if constexpr (SPLIT) {
        const int z = (int)blockIdx.z;
        const int c_first = z * c_lo + min(z, c_rem);
        const int c_count = c_lo + (z < c_rem ? 1 : 0);
        kt0 = (int64_t)c_first * CHUNK_TILES;
        a.n_kt = min(a.n_kt - kt0, (int64_t)c_count * CHUNK_TILES);
        a.K = a.n_kt * TILE_K;                               // (the rows keep their stride: see row_stride)
        a.xq += kt0 * TILE_K;
    } else {
        a.part = nullptr;
    }
    const int n_chunks = (int)((a.n_kt + CHUNK_TILES - 1) / CHUNK_TILES);
    const int c_b = 0, c_e = n_chunks;
    const int64_t kt_hi = a.n_kt;
    (void)n;

    int arow[RT];                                            // padded rows repeat the last
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) arow[rt] = (rt * 16 + l16 < rows ? rt * 16 + l16 : rows - 1) * ROW_STRIDE;

    // Dequant as in the tiled kernel: every group starts from BIAS = 2^21 (third MFMA operand), so
    // acc = BIAS + 64*sum is positive and below 2^23 and its bit pattern read as binary32 is the
    // denormal acc * 2^-149: y += as_float(acc) * (sw * 2^64) is ONE fma per accumulator, no
    // int->float conversion.  The bias term 2^-128 * (sum of the scaled scales) is taken out every
    // few tiles and at the end.  Two accumulator sets alternate between groups, and a finished
    // group is dequantised right after the next group's first matrix instructions have been
    // issued, so that the vector work runs under them.
    constexpr int BIAS = 1 << 21;                            // > 64 * 127 * 2 * 128
    const v4i biasv = {BIAS, BIAS, BIAS, BIAS};
    float y[RT][4];
    v4i acc[2][RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        acc[0][rt] = biasv;
        acc[1][rt] = biasv;
#pragma unroll
        for (int r = 0; r < 4; ++r) y[rt][r] = 0.f;
    }
    float ssum = 0.f;                                        // sum of sw * 2^64 over the groups folded into y
    float pend_sw = 0.f;                                     // the finished group waiting in acc[1]: none yet
    int64_t pend_g = 0;

    // Activation chunks -> registers -> LDS.  Chunk c starts at k tile min(4c, n_kt - 4), so every
    // chunk is 1024 k wide (the last one overlaps its predecessor when K is not a multiple of 1024;
    // a K below 1024 is one narrower chunk) and a thread's pieces sit at the same offsets in every
    // chunk: piece i = 16 bytes, row i / 64, bytes 16 * (i % 64) of the row; both offsets are
    // computed once.  Every slot always loads (no branch around a load: with loads under a
    // condition the compiler cannot count how many are in flight, and its waits for older
    // registers then also wait for loads just issued): slots past the last row, and every slot
    // once there is no further chunk (real == false), re-read pieces of row 0.
    uint4 xs[NS];
    constexpr int VPR = CHUNK_TILES * TILE_K / 16;           // pieces per full row: 64
    const int64_t last_base = a.n_kt > CHUNK_TILES ? a.n_kt - CHUNK_TILES : 0;
    uint32_t goff[NS], loff[NS];
    {
        const int v_last = (int)min((int64_t)CHUNK_TILES, a.n_kt) * (TILE_K / 16) - 1;
#pragma unroll
        for (int j = 0; j < NS; ++j) {
            const unsigned i = threadIdx.x + j * THREADS;
            const unsigned row = i < (unsigned)(rows * VPR) ? i / VPR : 0;
            const unsigned v = min(i % VPR, (unsigned)v_last);
            goff[j] = row * (uint32_t)row_stride + v * 16;   // < 64 K: fits 32 bits (K <= 2^24)
            loff[j] = (i / VPR) * ROW_STRIDE + (i % VPR) * 16;
        }
    }
    auto chunk_base = [&](int c) { return min((int64_t)c * CHUNK_TILES, last_base); };
    auto load_x = [&](int c, bool real) {
        const int8_t* src = a.xq + (real ? chunk_base(c) : 0) * TILE_K;    // uniform
        // no further chunk: stay inside the first min(K, 1024) bytes of row 0 (x & m <= m)
        const uint32_t mask = real ? 0xffffffffu : (uint32_t)min((int64_t)CHUNK_TILES * TILE_K, a.K) - 16u;
#pragma unroll
        for (int j = 0; j < NS; ++j) {
            xs[j] = make_uint4(0, 0, 0, 0);                  // (a dead store that keeps xs in registers)
            uint32_t off = goff[j] & mask;
            asm volatile("" : "+v"(off));                    // keeps "scalar base + 32-bit offset" addressing
            xs[j] = *reinterpret_cast<const uint4*>(src + off);
        }
        __builtin_amdgcn_sched_barrier(0);                   // the loads stay here, ahead of the arithmetic
    };
    auto store_x = [&]() {
#pragma unroll
        for (int j = 0; j < NS; ++j)
            if (threadIdx.x + j * THREADS < (unsigned)(rows * VPR)) *reinterpret_cast<uint4*>(smem + loff[j]) = xs[j];
    };
    // tile s of this wave is k tile ks + s*KS; its address is a wave-uniform base plus a 32-bit
    // lane offset, so the loads need no vector address arithmetic
    uint32_t w_lane = (uint32_t)lane * 16u, s_lane = (uint32_t)l16 * (GPT * 2u);
    auto load_w = [&](int64_t s) {
        int64_t kt = ks + s * KS;
        kt = kt < kt_hi ? kt : kt_hi - 1;                    // past this workgroup's range: its last tile again
        const int64_t tile = cbc * kt_stride + kt0 + kt;
        const char* wbase = reinterpret_cast<const char*>(a.codes) + tile * (TILE_N * TILE_K / 4);
        const char* sbase = reinterpret_cast<const char*>(a.scales) + tile * (TILE_N * GPT * 2);
        asm volatile("" : "+v"(w_lane), "+v"(s_lane));
        TileRegs r;
        r.w = *reinterpret_cast<const uint4*>(wbase + w_lane);
        if constexpr (G == 128) {
            r.s0 = *reinterpret_cast<const uint32_t*>(sbase + s_lane);
            r.s1 = 0;
        } else {
            const uint2 sc = *reinterpret_cast<const uint2*>(sbase + s_lane);
            r.s0 = sc.x; r.s1 = sc.y;
        }
        return r;
    };
    // y += as_float(acc[b]) * sw for the group waiting in accumulator set b
    auto dequant = [&](int b) {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if constexpr (DBG) {
                    const int m = rt * 16 + 4 * q + r;
                    if (pend_sw != 0.f && cb_ok && n < a.N && m < a.M)
                        a.acc_out[((int64_t)m * (a.K / G) + pend_g) * a.N + n] = (acc[b][rt][r] - BIAS) >> 6;
                }
                y[rt][r] = fmaf(__int_as_float(acc[b][rt][r]), pend_sw, y[rt][r]);
            }
        ssum += pend_sw;
    };
    auto compute = [&](const TileRegs& cur, int64_t kt, int kt_in_chunk) {
        const int8_t* xk = smem + kt_in_chunk * TILE_K + q * 16;
        const uint32_t wd[4] = {cur.w.x, cur.w.y, cur.w.z, cur.w.w};
        v4i aop[2][RT];                                      // A operands of this 64-k step and the next
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) aop[0][rt] = *reinterpret_cast<const v4i*>(xk + arow[rt]);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            if (t < 3) {
#pragma unroll
                for (int rt = 0; rt < RT; ++rt)
                    aop[(t + 1) & 1][rt] = *reinterpret_cast<const v4i*>(xk + arow[rt] + (t + 1) * 64);
            }
            int u[4];
            upconvert(wd[t], u);
            const v4i bop = {u[0], u[1], u[2], u[3]};
            const int gi = G == 64 ? t : t >> 1;             // group inside the tile
            const int b = gi & 1;                            // its accumulator set
            const bool first = G == 64 || !(t & 1);
            const bool last = G == 64 || (t & 1);
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
                acc[b][rt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(aop[t & 1][rt], bop, first ? biasv : acc[b][rt], 0, 0, 0);
            if (first) dequant(b ^ 1);                       // the group before this one, under these MFMAs
            if (last) {
                pend_sw = DBG ? 1.0f : tile_scale<G>(cur, gi) * 0x1p64f;
                pend_g = kt * GPT + gi;
            }
        }
    };
    // take the accumulated bias term out of y (keeps the rounding error near 2^-15 of the result)
    auto settle = [&]() {
        const float corr = ssum * 0x1p-128f;                 // BIAS * 2^-149 = 2^-128
        ssum = 0.f;
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int r = 0; r < 4; ++r) y[rt][r] -= corr;
    };

    // activation loads first, then the weight window: vector memory returns in order, so the
    // wait for the activations does not wait for the weights behind them
    load_x(c_b, true);
    TileRegs tr[D];
    const int64_t s_b = (int64_t)c_b * TPC, s_e = (int64_t)c_e * TPC;    // the same for every wave: barriers match
#pragma unroll
    for (int i = 0; i < D; ++i) tr[i] = load_w(s_b + i);
    __builtin_amdgcn_sched_barrier(0);

    for (int64_t s0 = s_b; s0 < s_e; s0 += D) {
#pragma unroll
        for (int i = 0; i < D; ++i) {
            const int64_t s = s0 + i;
            const int c = (int)(s / TPC);
            if (i % TPC == 0) {
                if (c >= c_e) break;
                if (c > c_b) __syncthreads();                // everyone is done reading chunk c-1
                store_x();
                __syncthreads();
                load_x(c + 1, c + 1 < c_e);
            }
            const int64_t kt = ks + s * KS;
            if (kt < kt_hi) compute(tr[i], kt, (int)(kt - chunk_base(c)));
            if ((i & 3) == 3) settle();                      // every 8 (G=128) or 16 (G=64) groups
            tr[i] = load_w(s + D);                           // past the end: re-reads the last tile
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    dequant(1);                                             // the last group (GPT is even: it sits in set 1)
    if constexpr (DBG) return;
    settle();

    __syncthreads();                                        // activations no longer needed
    float* red = reinterpret_cast<float*>(smem);            // [waves][16*RT m][16 n]
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int r = 0; r < 4; ++r) red[((wave * RT + rt) * 16 + 4 * q + r) * 16 + l16] = y[rt][r] * 0x1p79f;   // 2^(149-64-6)
    __syncthreads();
    if (a.part) {
        // this K range's share of the result, as fp32 [m][n] rows of the workspace (16 * CBW adjacent
        // columns per row); a second launch adds the ranges in a fixed order and applies the epilogue
        for (int i = threadIdx.x; i < CBW * rows * 16; i += THREADS) {
            const int nl = i & 15, ci = (i >> 4) % CBW, m = i / (16 * CBW);
            const int64_t nn = ((int64_t)blockIdx.x * CBW + ci) * TILE_N + nl;
            if (nn >= a.N) continue;
            float s = 0.0f;
#pragma unroll
            for (int k = 0; k < KS; ++k) s += red[((k * CBW + ci) * (RT * 16) + m) * 16 + nl];
            a.part[(int64_t)m * a.N + nn] = s * a.sx[m];
        }
        return;
    }
    store_outputs(a.epi, a.Y, a.ldy, a.N, (int64_t)blockIdx.x * CBW, CBW, rows,
                  [&](int ci, int m, int nl, int) {
                      float s = 0.0f;
#pragma unroll
                      for (int k = 0; k < KS; ++k) s += red[((k * CBW + ci) * (RT * 16) + m) * 16 + nl];
                      return s * a.sx[m];
                  });
}

template <int G, int RT, int TPC>
static int launch_t(const A8Args& a_in, int splits, hipStream_t stream)
{
    constexpr int CBW = 2 * TPC;
    A8Args a = a_in;
    if (splits < 2 || a.acc_out) { a.part = nullptr; splits = 1; }
    const int64_t band = a.M < ROWS_PER_BAND ? a.M : ROWS_PER_BAND;
    const size_t act = (size_t)band * ROW_STRIDE;
    const size_t red = (size_t)8 * RT * 16 * 16 * sizeof(float);
    const size_t lds = act > red ? act : red;
    const int n_chunks = (int)((a.n_kt + CHUNK_TILES - 1) / CHUNK_TILES);
    const dim3 grid((unsigned)((a.n_cb + CBW - 1) / CBW), (unsigned)((a.M + ROWS_PER_BAND - 1) / ROWS_PER_BAND),
                    (unsigned)splits), block(THREADS);
    auto go = [&](auto kern) {
        if (int rc = ensure_dynamic_lds((const void*)kern, lds, "w2_matmul_a8[midm]")) return rc;
        hipLaunchKernelGGL(kern, grid, block, lds, stream, a, n_chunks / splits, n_chunks % splits);
        return check_launch("w2_matmul_a8[midm]");
    };
    if (a.acc_out) return go(a8_midm_kernel<G, RT, TPC, true, false>);
    if (splits < 2) return go(a8_midm_kernel<G, RT, TPC, false, false>);
    if (int rc = go(a8_midm_kernel<G, RT, TPC, false, true>)) return rc;
    return launch_splitk_reduce(a.part, splits, a.M, a.N, a.Y, a.ldy, a.epi, stream);
}

template <int G, int RT>
static int launch_rt(const A8Args& a, hipStream_t stream)
{
    const int64_t cap = a.part ? (int64_t)(a.part_bytes / ((size_t)a.M * a.N * sizeof(float))) : 0;
    const MidmPlan p = midm_plan(a.M, a.n_cb, a.n_kt, cap, a.tune);
    if (p.cbw == 8) return launch_t<G, RT, 4>(a, p.splits, stream);
    if (p.cbw == 4) return launch_t<G, RT, 2>(a, p.splits, stream);
    return launch_t<G, RT, 1>(a, p.splits, stream);
}

template <int G>
static int launch_g(const A8Args& a, hipStream_t stream)
{
    if (a.M <= 16) return launch_rt<G, 1>(a, stream);
    if (a.M <= 32) return launch_rt<G, 2>(a, stream);
    return launch_rt<G, 4>(a, stream);                       // eight row tiles would not fit the registers
}

}  // namespace midm

// up to four bands of 64 rows (beyond that the tiled kernel's reuse of the weights wins everywhere)
bool a8_midm_supports(const A8Args& a) { return a.M >= 1 && a.M <= 4 * midm::ROWS_PER_BAND; }

size_t a8_midm_splitk_bytes(int64_t M, int64_t N, int64_t n_cb, int64_t n_kt, const w2_tuning_t& tune)
{
    const int s = midm_plan(M, n_cb, n_kt, 16, tune).splits;
    return s < 2 ? 0 : (size_t)s * M * N * sizeof(float);
}

int launch_a8_midm(const A8Args& a, hipStream_t stream)
{
    return a.G == 128 ? midm::launch_g<128>(a, stream) : midm::launch_g<64>(a, stream);
}

}  // namespace w2
