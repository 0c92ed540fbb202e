// w2a8 with the activation quantisation fused into the matmul kernel, for
// M <= 4 (Sec. II-D: on a GPU the separate quantise -> GEMM -> dequantise
// sequence costs launches and passes, so the paper's kernel takes 16/32-bit
// activations, computes the abs-max per workgroup -- redundantly, every
// workgroup repeats it -- keeps it in local memory, quantises in the kernel
// and dequantises before the store; Sec. III-C reports that fusing wins for
// matrix-vector shapes).  Arithmetic of the quantisation is that of
// w2_quantize_rows, operation for operation, so the int8 codes and the
// result are bit-identical to the two-call path.
//
// Built on the small-M MFMA kernel: each workgroup loads the M activation
// rows (vector loads issued before the weight loads) into registers,
// reduces abs-max across its waves, quantises them into the int8 rows (LDS) the
// matrix instructions read.  No vector memory is touched between the weight
// loads and their first use, so nothing waits behind the weight stream.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "w2_small_common.h"

namespace w2 {

constexpr int FQ_HDR = 512;       // bytes: abs-max partials [16 waves][4 rows], then sx[4]
constexpr int FQ_PIECES = 8;      // 16-byte pieces of the activation rows per thread (registers)

__device__ __forceinline__ int fq_quant1(float x, float inv)
{
    float t = x * inv;                        // one rounded multiply
    float r = __builtin_rintf(t);             // half to even
    r = fminf(fmaxf(r, -127.0f), 127.0f);
    return (int)r;
}

__device__ __forceinline__ uint32_t fq_pack4(int a, int b, int c, int d)
{
    return (a & 0xff) | ((b & 0xff) << 8) | ((c & 0xff) << 16) | ((uint32_t)(d & 0xff) << 24);
}

struct FusedArgs {
    const uint32_t* codes;
    const uint16_t* scales;
    const void* X;
    uint16_t* Y;
    int64_t M, K, N, ldx, ldy;
    int64_t n_cb, n_kt;
    int G;
    Epilogue epi;
};

template <int G, int TMAX, int RL, bool BF16IN, int PRE = TMAX>
__global__ void __launch_bounds__(1024)
a8_fusedq_kernel(FusedArgs a, SmallCfg cfg)
{
    W2_SMALL_PROLOGUE();
    (void)cb_ok; (void)n_chunks; (void)tiles_per_chunk;
    const int rows = (int)a.M;                              // 1..4
    const int arow = (lane & 15) < rows ? (lane & 15) : rows - 1;
    constexpr int ES = BF16IN ? 2 : 4;                      // bytes per source element
    constexpr int EPP = 16 / ES;                            // elements per 16-byte piece
    const int K = (int)a.K;
    const int ppr = K / EPP;                                // pieces per row
    const int total = rows * ppr;
    const int row_stride = K + XS_PAD;
    float* s_red = reinterpret_cast<float*>(smem);          // [16][4]
    float* s_sx = s_red + 64;                               // [4]
    int8_t* xs = smem + FQ_HDR;                             // int8 rows

    // piece index -> (row, piece inside the row); a single row needs no division
    auto split = [&](unsigned i, int& r, int& v) __attribute__((always_inline)) {
        if constexpr (RL == 1) { r = 0; v = (int)i; }
        else { r = (int)(i / (unsigned)ppr); v = (int)i - r * ppr; }
    };

    // 1. activation rows: vector loads first
    uint4 pc[FQ_PIECES];
#pragma unroll
    for (int j = 0; j < FQ_PIECES; ++j) {
        // slots wholly past the end are skipped (uniform branch); surplus threads of the last slot
        // re-read pieces spread over the rows, never one common cache line
        pc[j] = make_uint4(0, 0, 0, 0);
        if (j * (int)blockDim.x < total) {
            unsigned i = threadIdx.x + j * blockDim.x;
            if (i >= (unsigned)total) i %= (unsigned)total;     // only the lanes past the end pay for the division
            int r, v;
            split(i, r, v);
            pc[j] = *reinterpret_cast<const uint4*>((const char*)a.X + ((int64_t)r * a.ldx * ES) + (int64_t)v * 16);
        }
    }
    // 2. the wave's whole share of the weight stream
    int64_t kt0 = ks;
    const int64_t kt_end = a.n_kt;
    auto load_range = [&](int64_t kb, TileRegs (&tr)[TMAX], auto first, auto last) {
#pragma unroll
        for (int i = decltype(first)::value; i < decltype(last)::value; ++i) {
            const int64_t kt = kb + (int64_t)i * cfg.ks;
            tr[i] = load_tile<G>(a.codes, a.scales, cbc * a.n_kt + (kt < kt_end ? kt : kt_end - 1), lane);
        }
    };
    auto load_batch = [&](int64_t kb, TileRegs (&tr)[TMAX]) {
        load_range(kb, tr, std::integral_constant<int, 0>{}, std::integral_constant<int, TMAX>{});
    };
    // Only the first PRE tiles are requested before the activations are quantised.  With every
    // load of a large projection issued up front the memory pipeline fills, the waves stall in
    // the issue of their later loads, and the barriers below (hence the first matrix instruction)
    // wait for the slowest of them: measured with in-kernel timestamps on 4096 x 28672, the
    // quantised row was ready after 4.6 us (median over the waves) and most arithmetic ran
    // after the weights had arrived; with the split it is ready after 3.2 us.  The first tiles
    // keep the memory system busy while the rows are quantised; the rest is requested right after.
    TileRegs tr0[TMAX];
    load_range(kt0, tr0, std::integral_constant<int, 0>{}, std::integral_constant<int, PRE>{});

    // 3. reduce abs-max per row; the pieces stay in registers (every piece has a slot: a launch condition)
    float amax[RL];
#pragma unroll
    for (int rr = 0; rr < RL; ++rr) amax[rr] = 0.f;
#pragma unroll
    for (int j = 0; j < FQ_PIECES; ++j) {
        const int i = threadIdx.x + j * blockDim.x;
        if (i < total) {
            int r, v_unused;
            split((unsigned)i, r, v_unused);
            const uint32_t d[4] = {pc[j].x, pc[j].y, pc[j].z, pc[j].w};
            float m = 0.f;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if constexpr (BF16IN) {
                    m = fmaxf(m, fabsf(__uint_as_float(d[e] << 16)));
                    m = fmaxf(m, fabsf(__uint_as_float(d[e] & 0xffff0000u)));
                } else {
                    m = fmaxf(m, fabsf(__uint_as_float(d[e])));
                }
            }
#pragma unroll
            for (int rr = 0; rr < RL; ++rr) amax[rr] = (rr == r) ? fmaxf(amax[rr], m) : amax[rr];
        }
    }
#pragma unroll
    for (int rr = 0; rr < RL; ++rr) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) amax[rr] = fmaxf(amax[rr], __shfl_xor(amax[rr], off));
    }
    if (lane == 0) {
#pragma unroll
        for (int rr = 0; rr < RL; ++rr) s_red[wave * 4 + rr] = amax[rr];
    }
    __syncthreads();
    const int n_waves = blockDim.x >> 6;
    float inv[RL], sxv[RL];
#pragma unroll
    for (int rr = 0; rr < RL; ++rr) {
        float m = 0.f;
        for (int w = 0; w < n_waves; ++w) m = fmaxf(m, s_red[w * 4 + rr]);
        inv[rr] = 0.f; sxv[rr] = 0.f;
        if (m > 0.f) {
            inv[rr] = __fdiv_rn(127.0f, m);
            sxv[rr] = __fdiv_rn(m, 127.0f);
        }
    }
#pragma unroll
    for (int rr = 0; rr < RL; ++rr)
        if (threadIdx.x == (unsigned)rr) s_sx[rr] = sxv[rr];

    // 4. quantise the pieces into the int8 rows
#pragma unroll
    for (int j = 0; j < FQ_PIECES; ++j) {
        const int i = threadIdx.x + j * blockDim.x;
        if (i < total) {
            const uint4 p = pc[j];
            int r, v;
            split((unsigned)i, r, v);
            float iv = inv[0];
#pragma unroll
            for (int rr = 1; rr < RL; ++rr) iv = (r == rr) ? inv[rr] : iv;
            const uint32_t d[4] = {p.x, p.y, p.z, p.w};
            if constexpr (BF16IN) {
                int qv[8];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    qv[2 * e] = fq_quant1(__uint_as_float(d[e] << 16), iv);
                    qv[2 * e + 1] = fq_quant1(__uint_as_float(d[e] & 0xffff0000u), iv);
                }
                *reinterpret_cast<uint2*>(xs + r * row_stride + v * 8) =
                    make_uint2(fq_pack4(qv[0], qv[1], qv[2], qv[3]), fq_pack4(qv[4], qv[5], qv[6], qv[7]));
            } else {
                *reinterpret_cast<uint32_t*>(xs + r * row_stride + v * 4) =
                    fq_pack4(fq_quant1(__uint_as_float(d[0]), iv), fq_quant1(__uint_as_float(d[1]), iv),
                             fq_quant1(__uint_as_float(d[2]), iv), fq_quant1(__uint_as_float(d[3]), iv));
            }
        }
    }
    __syncthreads();
    load_range(kt0, tr0, std::integral_constant<int, PRE>{}, std::integral_constant<int, TMAX>{});

    // 5. up-convert and compute, as in the small-M kernel
    float y[RL];
#pragma unroll
    for (int r = 0; r < RL; ++r) y[r] = 0.f;
    // Two accumulators alternate between groups, and a finished group is dequantised one group
    // later, after the next group's matrix instructions have been issued: the int -> float
    // conversion then never waits for the matrix pipe, and the next tile's activation operands
    // are read from LDS while this tile is multiplied.  What a wave does after its last tile has
    // arrived is the kernel's tail, so the length of this chain counts.
    v4i acc[2] = {{0, 0, 0, 0}, {0, 0, 0, 0}};
    float pend_sw = 0.f;                                     // scale of the group waiting in acc[1]: none yet
    auto dequant = [&](int b) {
#pragma unroll
        for (int r = 0; r < RL; ++r) y[r] = fmaf(pend_sw, (float)acc[b][r], y[r]);
    };
    auto read_aop = [&](int64_t kt, v4i (&aop)[4]) {
        const int8_t* xrow = xs + arow * row_stride + (int)kt * TILE_K + q * 16;
#pragma unroll
        for (int t = 0; t < 4; ++t) aop[t] = *reinterpret_cast<const v4i*>(xrow + t * 64);
    };
    auto compute_batch = [&](int64_t kb, const TileRegs (&tr)[TMAX]) {
        v4i aop[2][4];
        read_aop(min(kb, kt_end - 1), aop[0]);
#pragma unroll
        for (int i = 0; i < TMAX; ++i) {
            const int64_t kt = kb + (int64_t)i * cfg.ks;
            if (kt >= kt_end) break;
            if (i + 1 < TMAX) read_aop(min(kt + cfg.ks, kt_end - 1), aop[(i + 1) & 1]);   // clamped: stays inside the rows
            __builtin_amdgcn_sched_barrier(0);               // the reads stay here, a tile ahead of their use
            const TileRegs cur = tr[i];
            const uint32_t wd[4] = {cur.w.x, cur.w.y, cur.w.z, cur.w.w};
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                int u[4];
                upconvert(wd[t], u);
                const v4i bop = {u[0], u[1], u[2], u[3]};
                const int gi = G == 64 ? t : t >> 1;         // group inside the tile
                const int b = gi & 1;                        // its accumulator (groups per tile are even)
                const bool first = G == 64 || !(t & 1);
                const v4i zero = {0, 0, 0, 0};
                acc[b] = __builtin_amdgcn_mfma_i32_16x16x64_i8(aop[i & 1][t], bop, first ? zero : acc[b], 0, 0, 0);
                if (first) {
                    __builtin_amdgcn_sched_barrier(0);       // ... after this group's first matrix instruction, not before
                    dequant(b ^ 1);                          // the group before this one
                }
                if (G == 64 || (t & 1)) pend_sw = tile_scale<G>(cur, gi);
            }
        }
    };
    compute_batch(kt0, tr0);
    for (kt0 += (int64_t)TMAX * cfg.ks; kt0 < kt_end; kt0 += (int64_t)TMAX * cfg.ks) {
        TileRegs tr[TMAX];
        load_batch(kt0, tr);
        compute_batch(kt0, tr);
    }
    dequant(1);                                              // the last group (it sits in acc[1])

    __syncthreads();
    float* red = reinterpret_cast<float*>(smem + FQ_HDR);   // [waves][16 m][16 n]
#pragma unroll
    for (int r = 0; r < RL; ++r) red[(wave * 16 + 4 * q + r) * 16 + (lane & 15)] = y[r];
    __syncthreads();
    store_outputs(a.epi, a.Y, a.ldy, a.N, (int64_t)blockIdx.x * cfg.cbw, cfg.cbw, rows,
                  [&](int ci, int m, int nl, int) {
                      float s = 0.0f;
                      for (int k = 0; k < cfg.ks; ++k) s += red[((k * cfg.cbw + ci) * 16 + m) * 16 + nl];
                      return s * (s_sx[m] * 0.015625f);
                  });
}

template <int G, int RL, bool BF16IN>
static int launch_fusedq_t(const FusedArgs& a, const SmallCfg& c, size_t lds, int pre, hipStream_t stream)
{
    const int tpw = (int)((a.n_kt + c.ks - 1) / c.ks);
    const char* what = "w2_matmul_a8_fused";
    if (tpw <= 2) return launch_small(a8_fusedq_kernel<G, 2, RL, BF16IN>, what, a, c, lds, stream);
    if (tpw <= 4) return launch_small(a8_fusedq_kernel<G, 4, RL, BF16IN>, what, a, c, lds, stream);
    // every wave has more than four tiles: a large projection.  One row: half of the loads wait for
    // the quantised row (measured 10.0 against 10.4 us on 4096 x 28672; with two rows it loses).
    if (RL == 1 && pre != 8)
        return launch_small(a8_fusedq_kernel<G, TMAX, RL, BF16IN, 4>, what, a, c, lds, stream);
    return launch_small(a8_fusedq_kernel<G, TMAX, RL, BF16IN>, what, a, c, lds, stream);
}

// Returns -2 (unsupported shape) with a message if the rows do not fit the
// per-workgroup budget; the caller then uses w2_quantize_rows + w2_matmul_a8.
int launch_a8_fusedq(const void* codes, const void* scales, const void* X, int x_is_bf16, int64_t ldx,
                     int64_t M, int64_t K, int64_t N, int G, int64_t n_cb, int64_t n_kt, uint16_t* Y,
                     int64_t ldy, const Epilogue& epi, const w2_tuning_t& tune, hipStream_t stream)
{
    if (M < 1 || M > 4) {
        set_error("w2_matmul_a8_fused: M must be 1..4 (use w2_quantize_rows + w2_matmul_a8)");
        return -2;
    }
    const int rows = (int)M;
    const int es = x_is_bf16 ? 2 : 4;
    const int64_t pieces = M * K * es / 16;                  // every piece needs a register slot of some thread
    SmallCfg c = pick_cfg(tune, n_cb, n_kt, rows, 1, 16, epi.act == ACT_SILU_MUL, (int)((pieces + FQ_PIECES - 1) / FQ_PIECES));
    const int threads = 64 * c.cbw * c.ks;
    const size_t xs_bytes = ((size_t)rows * (K + XS_PAD) + 15) & ~(size_t)15;
    size_t lds = FQ_HDR + xs_bytes;
    const size_t red = FQ_HDR + (size_t)c.cbw * c.ks * 16 * 16 * sizeof(float);
    if (red > lds) lds = red;
    if (c.kc != n_kt * TILE_K || pieces > (int64_t)FQ_PIECES * threads || lds > 144 * 1024) {
        set_error("w2_matmul_a8_fused: M*K too large for the fused path (use w2_quantize_rows + w2_matmul_a8)");
        return -2;
    }
    FusedArgs a;
    a.codes = (const uint32_t*)codes; a.scales = (const uint16_t*)scales; a.X = X; a.Y = Y;
    a.M = M; a.K = K; a.N = N; a.ldx = ldx; a.ldy = ldy; a.n_cb = n_cb; a.n_kt = n_kt; a.G = G;
    a.epi = epi;
    const int rl = M <= 1 ? 1 : M <= 2 ? 2 : 4;
#define W2_FQ(GG, RLL)                                                                         \
    return x_is_bf16 ? launch_fusedq_t<GG, RLL, true>(a, c, lds, tune.fused_pre, stream)       \
                     : launch_fusedq_t<GG, RLL, false>(a, c, lds, tune.fused_pre, stream)
    if (G == 128) {
        if (rl == 1) { W2_FQ(128, 1); }
        if (rl == 2) { W2_FQ(128, 2); }
        W2_FQ(128, 4);
    }
    if (rl == 1) { W2_FQ(64, 1); }
    if (rl == 2) { W2_FQ(64, 2); }
    W2_FQ(64, 4);
#undef W2_FQ
}

}  // namespace w2
