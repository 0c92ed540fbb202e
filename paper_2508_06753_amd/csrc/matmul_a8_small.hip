// w2a8 for small M (decode): the memory-bound regime where time tracks the
// bytes of weight streamed (Sec. I, II-A).  "Up-convert and compute"
// (Sec. II-C): each lane reads 128 bits of packed 2-bit weights, turns them
// into int8 operands in registers with one shift + one mask per four weights,
// and feeds int8 x int8 -> int32 instructions.  Two kernel families:
//   DOT4   v_dot4_i32_i8 per lane (the CDNA analog of the VNNI FMA microkernel
//          of Sec. II-C), M <= 4;
//   SMALLM one v_mfma_i32_16x16x64_i8 per 64-k step with the M rows padded to
//          the 16-row tile, M <= 16: the up-convert cost no longer grows with M.
// Both split K across the waves of a workgroup (Sec. II-D mentions K-splitting
// for small shapes) and reduce through LDS in a fixed order, so results are
// deterministic.  The dequant epilogue (Sec. II-D: int32 -> float, x scales,
// -> bf16) is fused: per group y += sw * float(acc), at the end y * sx / 64.
#include <hip/hip_runtime.h>

#include "w2_small_common.h"

namespace w2 {


// Staging of the activation rows [0,rows) x k in [k0, k0+len) into LDS rows of
// stride len + XS_PAD (len % 16 == 0), split in two so that the global loads
// can be issued BEFORE the weight-tile loads and the LDS stores after them:
// vector memory returns in order, so waiting for the activations then does
// not wait for the weights behind them.  Up to SV 16-byte pieces per thread go
// through registers; anything beyond that is copied directly.
constexpr int SV = 4;

struct StageRegs { uint4 v0, v1, v2, v3; };

__device__ __forceinline__ uint4 stage_load1(const int8_t* __restrict__ xq, int64_t K, int64_t k0,
                                             int vec_per_row, int total, int j)
{
    // A slot that lies wholly past the end is skipped (uniform branch).  Inside the last,
    // partly filled slot the surplus threads re-read pieces spread over the rows (i mod total):
    // if they all re-read one piece, every workgroup of the grid hammers the same cache line.
    uint4 r = make_uint4(0, 0, 0, 0);
    if (j * (int)blockDim.x < total) {
        unsigned i = threadIdx.x + j * blockDim.x;
        i = i < (unsigned)total ? i : i % (unsigned)total;
        const int row = i / vec_per_row, v = i - row * vec_per_row;
        r = *reinterpret_cast<const uint4*>(xq + (int64_t)row * K + k0 + v * 16);
    }
    return r;
}

__device__ __forceinline__ void stage_load(const int8_t* __restrict__ xq, int64_t K, int rows,
                                           int64_t k0, int len, StageRegs& st)
{
    const int vec_per_row = len >> 4;
    const int total = rows * vec_per_row;
    st.v0 = stage_load1(xq, K, k0, vec_per_row, total, 0);
    st.v1 = stage_load1(xq, K, k0, vec_per_row, total, 1);
    st.v2 = stage_load1(xq, K, k0, vec_per_row, total, 2);
    st.v3 = stage_load1(xq, K, k0, vec_per_row, total, 3);
}

__device__ __forceinline__ void stage_store1(int8_t* xs, int len, int vec_per_row, int total, int j,
                                             const uint4& val)
{
    const int i = threadIdx.x + j * blockDim.x;
    if (i < total) {
        const int r = i / vec_per_row, v = i - r * vec_per_row;
        *reinterpret_cast<uint4*>(xs + r * (len + XS_PAD) + v * 16) = val;
    }
}

__device__ __forceinline__ void stage_store(const int8_t* __restrict__ xq, int64_t K, int rows,
                                            int64_t k0, int len, const StageRegs& st, int8_t* xs)
{
    const int vec_per_row = len >> 4;
    const int total = rows * vec_per_row;
    stage_store1(xs, len, vec_per_row, total, 0, st.v0);
    stage_store1(xs, len, vec_per_row, total, 1, st.v1);
    stage_store1(xs, len, vec_per_row, total, 2, st.v2);
    stage_store1(xs, len, vec_per_row, total, 3, st.v3);
    for (int i = threadIdx.x + SV * blockDim.x; i < total; i += blockDim.x) {
        const int r = i / vec_per_row, v = i - r * vec_per_row;
        *reinterpret_cast<uint4*>(xs + r * (len + XS_PAD) + v * 16) =
            *reinterpret_cast<const uint4*>(xq + (int64_t)r * K + k0 + v * 16);
    }
}

// ---------------------------------------------------------------- DOT4
template <int MT, int G, int TMAX, bool DBG>
__global__ void __launch_bounds__(1024)
a8_dot4_kernel(A8Args a, SmallCfg cfg)
{
    W2_SMALL_PROLOGUE();
    const int rows = MT < (int)a.M ? MT : (int)a.M;
    // activation scale for the output this thread stores first, fetched before the stream starts
    const int m_first = (threadIdx.x >> 4) % rows;           // the row of this thread's first output
    const float sx_first = (!DBG && m_first < a.M) ? a.sx[m_first] : 0.0f;

    float y[MT];
    int acc[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) { y[m] = 0.0f; acc[m] = 0; }

    for (int c = 0; c < n_chunks; ++c) {
        const int64_t kt_begin = (int64_t)c * tiles_per_chunk;
        const int64_t kt_end = min(kt_begin + tiles_per_chunk, a.n_kt);
        // first tile of this wave inside the chunk: smallest kt >= kt_begin with kt % KS == ks
        int64_t kt0 = kt_begin + ((ks - kt_begin % cfg.ks) + cfg.ks) % cfg.ks;
        const int cur_stride = (int)(kt_end - kt_begin) * TILE_K + XS_PAD;
        auto load_batch = [&](int64_t kb, TileRegs (&tr)[TMAX]) {
#pragma unroll
            for (int i = 0; i < TMAX; ++i) {             // branch-free: past-the-end slots re-read the last tile
                const int64_t kt = kb + (int64_t)i * cfg.ks;
                tr[i] = load_tile<G>(a.codes, a.scales, cbc * a.n_kt + (kt < kt_end ? kt : kt_end - 1), lane);
            }
        };
        auto compute_batch = [&](int64_t kb, const TileRegs (&tr)[TMAX]) {
#pragma unroll
            for (int i = 0; i < TMAX; ++i) {
                const int64_t kt = kb + (int64_t)i * cfg.ks;
                if (kt >= kt_end) break;
                const TileRegs cur = tr[i];
                const int8_t* xrow = smem + (int)(kt - kt_begin) * TILE_K + q * 16;
                const uint32_t wd[4] = {cur.w.x, cur.w.y, cur.w.z, cur.w.w};
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    int u[4];
                    upconvert(wd[t], u);
#pragma unroll
                    for (int m = 0; m < MT; ++m) {
                        const int mr = m < rows ? m : rows - 1;
                        const v4i x = *reinterpret_cast<const v4i*>(xrow + mr * cur_stride + t * 64);
                        acc[m] = __builtin_amdgcn_sdot4(u[0], x[0], acc[m], false);
                        acc[m] = __builtin_amdgcn_sdot4(u[1], x[1], acc[m], false);
                        acc[m] = __builtin_amdgcn_sdot4(u[2], x[2], acc[m], false);
                        acc[m] = __builtin_amdgcn_sdot4(u[3], x[3], acc[m], false);
                    }
                    if (G == 64 || (t & 1)) {                   // a group ends here
                        const int gi = G == 64 ? t : t >> 1;
                        const float sw = tile_scale<G>(cur, gi);
#pragma unroll
                        for (int m = 0; m < MT; ++m) {
                            if constexpr (DBG) {
                                int s = acc[m];
                                s += __shfl_xor(s, 16);
                                s += __shfl_xor(s, 32);
                                if (q == 0 && cb_ok && n < a.N && m < a.M)
                                    a.acc_out[((int64_t)m * (a.K / G) + kt * GPT + gi) * a.N + n] = s >> 6;
                            }
                            y[m] = fmaf(sw, (float)acc[m], y[m]);
                            acc[m] = 0;
                        }
                    }
                }
            }
        };
        // first batch: activation loads, then weight loads, then the LDS stores
        {
            StageRegs st;
            stage_load(a.xq, a.K, rows, kt_begin * TILE_K, (int)(kt_end - kt_begin) * TILE_K, st);
            TileRegs tr[TMAX];
            load_batch(kt0, tr);
            if (c > 0) __syncthreads();          // everyone is done reading the previous chunk
            stage_store(a.xq, a.K, rows, kt_begin * TILE_K, (int)(kt_end - kt_begin) * TILE_K, st, smem);
            __syncthreads();
            compute_batch(kt0, tr);
        }
        for (kt0 += (int64_t)TMAX * cfg.ks; kt0 < kt_end; kt0 += (int64_t)TMAX * cfg.ks) {
            TileRegs tr[TMAX];
            load_batch(kt0, tr);
            compute_batch(kt0, tr);
        }
    }
    if constexpr (DBG) return;

    // cross-lane: the four k-blocks of a tile live in lanes l, l^16, l^32, l^48
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        y[m] += __shfl_xor(y[m], 16);
        y[m] += __shfl_xor(y[m], 32);
    }
    __syncthreads();                                        // activations no longer needed
    float* red = reinterpret_cast<float*>(smem);            // [waves][MT][16]
    if (q == 0) {
#pragma unroll
        for (int m = 0; m < MT; ++m) red[(wave * MT + m) * 16 + lane] = y[m];
    }
    __syncthreads();
    store_outputs(a.epi, a.Y, a.ldy, a.N, (int64_t)blockIdx.x * cfg.cbw, cfg.cbw, rows,
                  [&](int ci, int m, int nl, int i) {
                      float s = 0.0f;
                      for (int k = 0; k < cfg.ks; ++k) s += red[((k * cfg.cbw + ci) * MT + m) * 16 + nl];
                      const float sxm = i == (int)threadIdx.x ? sx_first : a.sx[m];
                      return s * (sxm * 0.015625f);
                  });
}

// ---------------------------------------------------------------- SMALLM (MFMA)
// RL = accumulator registers that hold live rows: the 16x16 result puts row 4*(lane>>4)+r in
// register r, so for M <= RL <= 4 only registers r < RL need the dequant step.
template <int G, int TMAX, int RL, bool DBG>
__global__ void __launch_bounds__(1024)
a8_smallm_kernel(A8Args a, SmallCfg cfg)
{
    W2_SMALL_PROLOGUE();
    const int rows = (int)a.M;                              // 1..16
    const int arow = (lane & 15) < rows ? (lane & 15) : rows - 1;   // padded rows repeat the last
    const float sx_first = DBG ? 0.0f : a.sx[(threadIdx.x >> 4) % rows];

    float y[RL];
#pragma unroll
    for (int r = 0; r < RL; ++r) y[r] = 0.f;
    // Two accumulators alternate between groups, and a finished group is dequantised one group
    // later, after the next group's first matrix instruction has been issued: the int -> float
    // conversion then does not wait for the matrix pipe, and the next tile's activation operands
    // are read from LDS while this tile is multiplied.  What a wave does after its last tile has
    // arrived is the kernel's tail, so the length of this chain counts (14336 x 4096 at M=1:
    // 7.5 -> 6.4 us in the fused kernel).
    v4i acc[2] = {{0, 0, 0, 0}, {0, 0, 0, 0}};
    float pend_sw = 0.f;                                     // scale of the group waiting in acc[1]: none yet
    int64_t pend_g = -1;                                     // its index (debug export)
    auto dequant = [&](int b) {
#pragma unroll
        for (int r = 0; r < RL; ++r) {
            if constexpr (DBG) {
                const int m = 4 * q + r;
                if (pend_g >= 0 && cb_ok && n < a.N && m < a.M)
                    a.acc_out[((int64_t)m * (a.K / G) + pend_g) * a.N + n] = acc[b][r] >> 6;
            }
            y[r] = fmaf(pend_sw, (float)acc[b][r], y[r]);
        }
    };

    for (int c = 0; c < n_chunks; ++c) {
        const int64_t kt_begin = (int64_t)c * tiles_per_chunk;
        const int64_t kt_end = min(kt_begin + tiles_per_chunk, a.n_kt);
        int64_t kt0 = kt_begin + ((ks - kt_begin % cfg.ks) + cfg.ks) % cfg.ks;
        const int cur_stride = (int)(kt_end - kt_begin) * TILE_K + XS_PAD;
        auto load_batch = [&](int64_t kb, TileRegs (&tr)[TMAX]) {
#pragma unroll
            for (int i = 0; i < TMAX; ++i) {             // branch-free: past-the-end slots re-read the last tile
                const int64_t kt = kb + (int64_t)i * cfg.ks;
                tr[i] = load_tile<G>(a.codes, a.scales, cbc * a.n_kt + (kt < kt_end ? kt : kt_end - 1), lane);
            }
        };
        auto read_aop = [&](int64_t kt, v4i (&aop)[4]) {
            const int8_t* xrow = smem + arow * cur_stride + (int)(kt - kt_begin) * TILE_K + q * 16;
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
                if (i + 1 < TMAX) read_aop(min(kt + cfg.ks, kt_end - 1), aop[(i + 1) & 1]);   // clamped: stays inside the chunk
                __builtin_amdgcn_sched_barrier(0);           // the reads stay here, a tile ahead of their use
                const TileRegs cur = tr[i];
                const uint32_t wd[4] = {cur.w.x, cur.w.y, cur.w.z, cur.w.w};
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    int u[4];
                    upconvert(wd[t], u);
                    const v4i bop = {u[0], u[1], u[2], u[3]};
                    const int gi = G == 64 ? t : t >> 1;     // group inside the tile
                    const int b = gi & 1;                    // its accumulator (groups per tile are even)
                    const bool first = G == 64 || !(t & 1);
                    const v4i zero = {0, 0, 0, 0};
                    acc[b] = __builtin_amdgcn_mfma_i32_16x16x64_i8(aop[i & 1][t], bop, first ? zero : acc[b], 0, 0, 0);
                    if (first) {
                        __builtin_amdgcn_sched_barrier(0);   // ... after this group's first matrix instruction, not before
                        dequant(b ^ 1);                      // the group before this one
                    }
                    if (G == 64 || (t & 1)) {
                        pend_sw = tile_scale<G>(cur, gi);
                        pend_g = kt * GPT + gi;
                    }
                }
            }
        };
        // first batch: activation loads, then weight loads, then the LDS stores
        {
            StageRegs st;
            stage_load(a.xq, a.K, rows, kt_begin * TILE_K, (int)(kt_end - kt_begin) * TILE_K, st);
            TileRegs tr[TMAX];
            load_batch(kt0, tr);
            if (c > 0) __syncthreads();          // everyone is done reading the previous chunk
            stage_store(a.xq, a.K, rows, kt_begin * TILE_K, (int)(kt_end - kt_begin) * TILE_K, st, smem);
            __syncthreads();
            compute_batch(kt0, tr);
        }
        for (kt0 += (int64_t)TMAX * cfg.ks; kt0 < kt_end; kt0 += (int64_t)TMAX * cfg.ks) {
            TileRegs tr[TMAX];
            load_batch(kt0, tr);
            compute_batch(kt0, tr);
        }
    }
    dequant(1);                                              // the last group (it sits in acc[1])
    if constexpr (DBG) return;

    __syncthreads();
    float* red = reinterpret_cast<float*>(smem);            // [waves][16 m][16 n]
#pragma unroll
    for (int r = 0; r < RL; ++r) red[(wave * 16 + 4 * q + r) * 16 + (lane & 15)] = y[r];
    __syncthreads();
    store_outputs(a.epi, a.Y, a.ldy, a.N, (int64_t)blockIdx.x * cfg.cbw, cfg.cbw, rows,
                  [&](int ci, int m, int nl, int i) {
                      float s = 0.0f;
                      for (int k = 0; k < cfg.ks; ++k) s += red[((k * cfg.cbw + ci) * 16 + m) * 16 + nl];
                      const float sxm = i == (int)threadIdx.x ? sx_first : a.sx[m];
                      return s * (sxm * 0.015625f);
                  });
}

// ---------------------------------------------------------------- host side

bool a8_dot4_supports(const A8Args& a) { return a.M >= 1 && a.M <= 4; }
bool a8_smallm_supports(const A8Args& a) { return a.M >= 1 && a.M <= 16; }

template <int MT, int G>
static int launch_dot4_t(const A8Args& a, hipStream_t stream)
{
    const int rows = MT < (int)a.M ? MT : (int)a.M;
    const SmallCfg c = pick_cfg(a.tune, a.n_cb, a.n_kt, rows, 1, 16, a.epi.act == ACT_SILU_MUL);
    const size_t lds = small_lds_bytes(c, rows, MT, 1, 0);
    if (a.acc_out) return launch_small(a8_dot4_kernel<MT, G, TMAX, true>, "w2_matmul_a8[dot4]", a, c, lds, stream);
    // in-flight depth = tiles per wave, so that no load slot re-reads a tile
    const int tpw = tiles_per_wave(a.n_kt, c);
    if (tpw <= 2) return launch_small(a8_dot4_kernel<MT, G, 2, false>, "w2_matmul_a8[dot4]", a, c, lds, stream);
    if (tpw <= 4) return launch_small(a8_dot4_kernel<MT, G, 4, false>, "w2_matmul_a8[dot4]", a, c, lds, stream);
    return launch_small(a8_dot4_kernel<MT, G, TMAX, false>, "w2_matmul_a8[dot4]", a, c, lds, stream);
}

int launch_a8_dot4(const A8Args& a, hipStream_t stream)
{
    const int mt = a.M <= 1 ? 1 : a.M <= 2 ? 2 : 4;
    if (a.G == 128) {
        if (mt == 1) return launch_dot4_t<1, 128>(a, stream);
        if (mt == 2) return launch_dot4_t<2, 128>(a, stream);
        return launch_dot4_t<4, 128>(a, stream);
    }
    if (mt == 1) return launch_dot4_t<1, 64>(a, stream);
    if (mt == 2) return launch_dot4_t<2, 64>(a, stream);
    return launch_dot4_t<4, 64>(a, stream);
}

template <int G, int RL>
static int launch_smallm_t(const A8Args& a, hipStream_t stream)
{
    const int rows = (int)a.M;
    const SmallCfg c = pick_cfg(a.tune, a.n_cb, a.n_kt, rows, 1, 16, a.epi.act == ACT_SILU_MUL);
    const size_t lds = small_lds_bytes(c, rows, 16, 1, 0);
    const int tpw = tiles_per_wave(a.n_kt, c);
    // the debug export runs the instantiation (in-flight depth, live rows) the same call without it would run
    if (a.acc_out) {
        if (tpw <= 2) return launch_small(a8_smallm_kernel<G, 2, RL, true>, "w2_matmul_a8[smallm]", a, c, lds, stream);
        if (tpw <= 4) return launch_small(a8_smallm_kernel<G, 4, RL, true>, "w2_matmul_a8[smallm]", a, c, lds, stream);
        return launch_small(a8_smallm_kernel<G, TMAX, RL, true>, "w2_matmul_a8[smallm]", a, c, lds, stream);
    }
    if (tpw <= 2) return launch_small(a8_smallm_kernel<G, 2, RL, false>, "w2_matmul_a8[smallm]", a, c, lds, stream);
    if (tpw <= 4) return launch_small(a8_smallm_kernel<G, 4, RL, false>, "w2_matmul_a8[smallm]", a, c, lds, stream);
    return launch_small(a8_smallm_kernel<G, TMAX, RL, false>, "w2_matmul_a8[smallm]", a, c, lds, stream);
}

int launch_a8_smallm(const A8Args& a, hipStream_t stream)
{
    const int rl = a.M <= 1 ? 1 : a.M <= 2 ? 2 : 4;
    if (a.G == 128) {
        if (rl == 1) return launch_smallm_t<128, 1>(a, stream);
        if (rl == 2) return launch_smallm_t<128, 2>(a, stream);
        return launch_smallm_t<128, 4>(a, stream);
    }
    if (rl == 1) return launch_smallm_t<64, 1>(a, stream);
    if (rl == 2) return launch_smallm_t<64, 2>(a, stream);
    return launch_smallm_t<64, 4>(a, stream);
}

}  // namespace w2
