// w2a16 for medium M (up to 64 rows): the weight stream is read exactly once,
// as in the w2a8 kernel for this range.  A wave owns one 16-column block and
// every KS-th 256-k tile of it, builds each dword's 16 weights once, as sw*q
// (the scale-folded 16-bit construction of Sec. II-D, "Alternative
// implementation": nothing to dequantise afterwards, one fp32 accumulator per
// output), and feeds them to RT row tiles of v_mfma_f32_16x16x32_bf16
// (M <= 16 RT).  K is split across the waves of a workgroup (Sec. II-D,
// K-splitting for small shapes) and reduced through LDS in a fixed order.
//
// Schedule: eight waves = CBW column blocks x KS k-splits.  The bf16 activations
// go through LDS in chunks of 1024 k (one buffer; the next chunk waits in
// registers while the current one is multiplied, and is stored between two
// barriers), de-interleaved [8 even k | 8 odd k] per 16-k block, the order in
// which the codes come out of a dword.  The weight tiles run through a rolling
// window of eight per wave.
#include <hip/hip_runtime.h>

#include "w2_small_common.h"

namespace w2 {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

namespace midm16 {

constexpr int THREADS = 512;
constexpr int CHUNK_TILES = 4;                                   // k tiles per LDS chunk
constexpr int ROW_STRIDE = CHUNK_TILES * TILE_K * 2 + 32;        // bytes per LDS activation row (32 mod 64: conflict-free operand reads)
constexpr int D = 8;                                             // weight tiles in flight per wave
constexpr int ROWS_PER_BAND = 64;                                // rows one workgroup multiplies (RT <= 4 row tiles)

// The four weights of one (group, column), low bytes and high bytes, indexed by the raw code
// (00 -> 0, 01 -> +sw, 10 -> -2 sw: sign flipped and exponent + 1, 11 -> -sw).
struct Lut { uint32_t lo4, hi4; };

__device__ __forceinline__ Lut make_lut(uint32_t s)              // s: bf16 bit pattern of the group scale
{
    const uint32_t neg = s ^ 0x8000u;
    const uint32_t neg2 = (s & 0x7f80u) ? ((s + 0x0080u) ^ 0x8000u) : neg;   // a zero scale stays (minus) zero
    const uint32_t a = s << 16;
    const uint32_t b = neg2 | (neg << 16);
    Lut l;
    l.lo4 = __builtin_amdgcn_perm(b, a, 0x06040200u);
    l.hi4 = __builtin_amdgcn_perm(b, a, 0x07050301u);
    return l;
}

// 16 codes of one dword -> b0 (even k of the lane's 16-k block), b1 (odd k)
__device__ __forceinline__ void upconvert16(uint32_t w, const Lut& l, v4i& b0, v4i& b1)
{
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t t = (w >> (2 * j)) & 0x03030303u;
        const uint32_t lo = __builtin_amdgcn_perm(0u, l.lo4, t);
        const uint32_t hi = __builtin_amdgcn_perm(0u, l.hi4, t);
        b0[j] = (int)__builtin_amdgcn_perm(hi, lo, 0x06020400u);
        b1[j] = (int)__builtin_amdgcn_perm(hi, lo, 0x07030501u);
    }
}

__device__ __forceinline__ v4f mfma_bf16(const v4i& a, const v4i& b, const v4f& c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf, a),
                                                   __builtin_bit_cast(v8bf, b), c, 0, 0, 0);
}

template <int G, int RT, int TPC, bool SPLIT>
__global__ void __launch_bounds__(THREADS)
a16_midm_kernel(A16Args a_all, int c_lo, int c_rem)
{
    // More than 64 rows: blockIdx.y picks a band of 64 rows; the bands stream the same weights (the
    // second one mostly out of L2), which pays when one band's workgroups would leave CUs idle.
    A16Args a = a_all;
    {
        const int64_t m_off = (int64_t)blockIdx.y * ROWS_PER_BAND;
        a.M = min((int64_t)ROWS_PER_BAND, a_all.M - m_off);
        a.X += m_off * a.ldx;
        a.Y += m_off * a.ldy;
        if (a.part) a.part += ((int64_t)blockIdx.z * a_all.M + m_off) * a.N;
    }
    constexpr int KS = CHUNK_TILES / TPC;                    // k-splits
    constexpr int CBW = 8 / KS;                              // column blocks per workgroup
    constexpr int VPR = CHUNK_TILES * TILE_K / 8;            // 16-byte pieces (eight k) per full row: 128
    constexpr int NS = RT * 16 * VPR / THREADS;              // pieces per thread and chunk: 4 RT
    constexpr int GPT = TILE_K / G;
    extern __shared__ __align__(16) int8_t smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int cbi = wave % CBW, ks = wave / CBW;
    const int q = lane >> 4, l16 = lane & 15;
    const int64_t cb = (int64_t)blockIdx.x * CBW + cbi;
    const int64_t cbc = cb < a.n_cb ? cb : a.n_cb - 1;       // clamp: keeps loads in bounds
    const int rows = (int)a.M;                               // 1..16*RT
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
        a.K = a.n_kt * TILE_K;                               // (the rows keep their stride ldx)
        a.X += kt0 * TILE_K;
    } else {
        a.part = nullptr;
    }
    const int n_chunks = (int)((a.n_kt + CHUNK_TILES - 1) / CHUNK_TILES);
    const int c_b = 0, c_e = n_chunks;
    const int64_t kt_hi = a.n_kt;
    if constexpr (!SPLIT) a.part = nullptr;

    int arow[RT];                                            // padded rows repeat the last
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) arow[rt] = (rt * 16 + l16 < rows ? rt * 16 + l16 : rows - 1) * ROW_STRIDE;

    v4f acc[2][RT];                                          // even-k and odd-k halves: two independent chains
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        acc[0][rt] = (v4f){0.f, 0.f, 0.f, 0.f};
        acc[1][rt] = (v4f){0.f, 0.f, 0.f, 0.f};
    }

    // Activation chunks -> registers -> LDS.  Chunk c starts at k tile min(4c, n_kt - 4), so every
    // chunk is 1024 k wide (the last one overlaps its predecessor when K is not a multiple of 1024;
    // a K below 1024 is one narrower chunk) and a thread's pieces sit at the same offsets in every
    // chunk: piece i = eight k, row i / 128, k 8 * (i % 128) of the chunk.  Every slot always loads
    // (no branch around a load, so the compiler's wait counts stay exact): slots past the last row,
    // and every slot once there is no further chunk, re-read pieces of row 0.
    uint4 xs[NS];
    const int64_t last_base = a.n_kt > CHUNK_TILES ? a.n_kt - CHUNK_TILES : 0;
    uint32_t goff[NS], loff[NS];
    {
        const int v_last = (int)min((int64_t)CHUNK_TILES, a.n_kt) * (TILE_K / 8) - 1;
#pragma unroll
        for (int j = 0; j < NS; ++j) {
            const unsigned i = threadIdx.x + j * THREADS;
            const unsigned row = i < (unsigned)(rows * VPR) ? i / VPR : 0;
            const unsigned v = min(i % VPR, (unsigned)v_last);
            goff[j] = row * (uint32_t)(a.ldx * 2) + v * 16;  // < 64 rows * 2 ldx: fits 32 bits (ldx <= 2^24)
            const unsigned vv = i % VPR;                     // 64-k block vv / 8, 16-k block (vv % 8) / 2, half vv % 2
            loff[j] = (i / VPR) * ROW_STRIDE + (vv >> 3) * 128 + ((vv & 7) >> 1) * 16 + (vv & 1) * 8;
        }
    }
    auto chunk_base = [&](int c) { return min((int64_t)c * CHUNK_TILES, last_base); };
    auto load_x = [&](int c, bool real) {
        const char* src = reinterpret_cast<const char*>(a.X) + (real ? chunk_base(c) : 0) * (TILE_K * 2);   // uniform
        // no further chunk: stay inside the first min(K, 1024) k of row 0 (x & m <= m)
        const uint32_t mask = real ? 0xffffffffu : (uint32_t)min((int64_t)CHUNK_TILES * TILE_K, a.K) * 2u - 16u;
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
            if (threadIdx.x + j * THREADS < (unsigned)(rows * VPR)) {
                const uint32_t d[4] = {xs[j].x, xs[j].y, xs[j].z, xs[j].w};
                uint2 ev, od;
                ev.x = __builtin_amdgcn_perm(d[1], d[0], 0x05040100u);
                ev.y = __builtin_amdgcn_perm(d[3], d[2], 0x05040100u);
                od.x = __builtin_amdgcn_perm(d[1], d[0], 0x07060302u);
                od.y = __builtin_amdgcn_perm(d[3], d[2], 0x07060302u);
                *reinterpret_cast<uint2*>(smem + loff[j]) = ev;
                *reinterpret_cast<uint2*>(smem + loff[j] + 64) = od;
            }
    };
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
    auto compute = [&](const TileRegs& cur, int kt_in_chunk) {
        const int8_t* xk = smem + kt_in_chunk * (TILE_K * 2) + q * 16;
        const uint32_t wd[4] = {cur.w.x, cur.w.y, cur.w.z, cur.w.w};
        v4i aop[2][RT];                                      // the operands of this 32-k step and the next
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) aop[0][rt] = *reinterpret_cast<const v4i*>(xk + arow[rt]);
        Lut lut = {0u, 0u};
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            if (G == 64 || !(t & 1)) {                       // a group begins
                const uint32_t pair = (G == 128 || t < 2) ? cur.s0 : cur.s1;
                const int hi = G == 128 ? t >> 1 : t & 1;
                lut = make_lut(hi ? pair >> 16 : pair & 0xffffu);
            }
            v4i b0, b1;
            upconvert16(wd[t], lut, b0, b1);
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int step = 2 * t + e;
                if (step < 7) {
#pragma unroll
                    for (int rt = 0; rt < RT; ++rt)
                        aop[(step + 1) & 1][rt] = *reinterpret_cast<const v4i*>(xk + arow[rt] + (step + 1) * 64);
                }
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) acc[e][rt] = mfma_bf16(aop[step & 1][rt], e == 0 ? b0 : b1, acc[e][rt]);
            }
        }
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
            if (kt < kt_hi) compute(tr[i], (int)(kt - chunk_base(c)));
            tr[i] = load_w(s + D);                           // past the end: re-reads the last tile
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    __syncthreads();                                        // activations no longer needed
    float* red = reinterpret_cast<float*>(smem);            // [waves][16*RT m][16 n]
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int r = 0; r < 4; ++r)
            red[((wave * RT + rt) * 16 + 4 * q + r) * 16 + l16] = acc[0][rt][r] + acc[1][rt][r];
    __syncthreads();
    if (a.part) {
        // this K range's share of the result, as fp32 [m][n] rows of the workspace; a second launch adds
        // the ranges in a fixed order and applies the epilogue
        for (int i = threadIdx.x; i < CBW * rows * 16; i += THREADS) {
            const int nl = i & 15, ci = (i >> 4) % CBW, m = i / (16 * CBW);
            const int64_t nn = ((int64_t)blockIdx.x * CBW + ci) * TILE_N + nl;
            if (nn >= a.N) continue;
            float s = 0.0f;
#pragma unroll
            for (int k = 0; k < KS; ++k) s += red[((k * CBW + ci) * (RT * 16) + m) * 16 + nl];
            a.part[(int64_t)m * a.N + nn] = s;
        }
        return;
    }
    store_outputs(a.epi, a.Y, a.ldy, a.N, (int64_t)blockIdx.x * CBW, CBW, rows,
                  [&](int ci, int m, int nl, int) {
                      float s = 0.0f;
#pragma unroll
                      for (int k = 0; k < KS; ++k) s += red[((k * CBW + ci) * (RT * 16) + m) * 16 + nl];
                      return s;
                  });
}

template <int G, int RT, int TPC>
static int launch_t(const A16Args& a_in, int splits, hipStream_t stream)
{
    constexpr int CBW = 2 * TPC;
    A16Args a = a_in;
    if (splits < 2) { a.part = nullptr; splits = 1; }
    const int64_t band = a.M < ROWS_PER_BAND ? a.M : ROWS_PER_BAND;
    const size_t act = (size_t)band * ROW_STRIDE;
    const size_t red = (size_t)8 * RT * 16 * 16 * sizeof(float);
    const size_t lds = act > red ? act : red;
    const int n_chunks = (int)((a.n_kt + CHUNK_TILES - 1) / CHUNK_TILES);
    const dim3 grid((unsigned)((a.n_cb + CBW - 1) / CBW), (unsigned)((a.M + ROWS_PER_BAND - 1) / ROWS_PER_BAND),
                    (unsigned)splits), block(THREADS);
    auto go = [&](auto kern) {
        if (int rc = ensure_dynamic_lds((const void*)kern, lds, "w2_matmul_a16[midm]")) return rc;
        hipLaunchKernelGGL(kern, grid, block, lds, stream, a, n_chunks / splits, n_chunks % splits);
        return check_launch("w2_matmul_a16[midm]");
    };
    if (splits < 2) return go(a16_midm_kernel<G, RT, TPC, false>);
    if (int rc = go(a16_midm_kernel<G, RT, TPC, true>)) return rc;
    return launch_splitk_reduce(a.part, splits, a.M, a.N, a.Y, a.ldy, a.epi, stream);
}

template <int G, int RT>
static int launch_rt(const A16Args& a, hipStream_t stream)
{
    // the same launch shape as the int8-activation kernel's (workgroup width, K ranges)
    const int64_t cap = a.part ? (int64_t)(a.part_bytes / ((size_t)a.M * a.N * sizeof(float))) : 0;
    const MidmPlan p = midm_plan(a.M, a.n_cb, a.n_kt, cap, a.tune);
    if (p.cbw == 8) return launch_t<G, RT, 4>(a, p.splits, stream);
    if (p.cbw == 4) return launch_t<G, RT, 2>(a, p.splits, stream);
    return launch_t<G, RT, 1>(a, p.splits, stream);
}

template <int G>
static int launch_g(const A16Args& a, hipStream_t stream)
{
    if (a.M <= 16) return launch_rt<G, 1>(a, stream);
    if (a.M <= 32) return launch_rt<G, 2>(a, stream);
    return launch_rt<G, 4>(a, stream);
}

}  // namespace midm16

// up to four bands of 64 rows
bool a16_midm_supports(const A16Args& a) { return a.M >= 1 && a.M <= 4 * midm16::ROWS_PER_BAND; }

size_t a16_midm_splitk_bytes(int64_t M, int64_t N, int64_t n_cb, int64_t n_kt, const w2_tuning_t& tune)
{
    const int s = midm_plan(M, n_cb, n_kt, 16, tune).splits;
    return s < 2 ? 0 : (size_t)s * M * N * sizeof(float);
}

int launch_a16_midm(const A16Args& a, hipStream_t stream)
{
    return a.G == 128 ? midm16::launch_g<128>(a, stream) : midm16::launch_g<64>(a, stream);
}

}  // namespace w2
