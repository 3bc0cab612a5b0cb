// Strided-batched B x B x B matmul over a block stack with a fused epilogue, for gfx950.
//
// This is the primitive the paper calls `bmm` (Sections 3.1, 4.1): every step of the
// hot path -- factor accumulation (Algorithm 1), the Newton-DB updates (Section 3.3),
// the Clenshaw recurrence (Appendix A.2) and the preconditioned update -- is this
// product with a different epilogue:
//     C_b = mult_b * (alpha * op(A_b) op(B_b) + beta * D_b + gamma * I)
//
// Design (CDNA4): one workgroup of 256 threads (four 64-wide wavefronts in a 2 x 2
// arrangement) owns one TM x TN output tile of one block.  K is walked in slabs of BK
// that go from global memory straight into LDS (global_load_lds_dwordx4: a wavefront-wide
// load fills 1 KB of LDS in lane order, every lane picks its own 16-byte source cell), two
// stages, the next slab in flight while the current one is multiplied.  Each wavefront
// accumulates its (TM/2) x (TN/2) sub-tile with v_mfma_f32_32x32x2_f32.
//
// Operand layouts.  An MFMA operand wants, per lane, the element (row = lane%32,
// k = lane/32).  Depending on which index is contiguous in global memory a slab is
// kept in one of two LDS layouts (a direct load cannot pad rows; cells are swizzled
// instead, by the choice of the source cell):
//   KC  [row][k]  (k contiguous; rows of BK floats, cell q of row r at q ^ swizzle(r)):
//       one 16-byte LDS read gives a lane its operand for four consecutive MFMAs
//       (k = 4*(lane/32) + s, s = 0..3);
//   RC  [k][row]  (row contiguous; k-lines of TILE floats, the 32-float halves of the
//       lines with bit 2 of k set swapped): four 4-byte reads, one per MFMA, lanes
//       reading consecutive addresses.
// Both layouts use the same k <-> (lane half, step) assignment, so any combination of
// transposed / non-transposed operands contracts over matching k.
//
// Grid.  1-D, one workgroup per (block, product, tile).  Hardware hands consecutive
// workgroup ids to the 8 XCDs round-robin; the id is remapped so that each XCD works
// through a contiguous range of blocks and the tiles of one block (which share the
// A and B panels) meet in one XCD's L2.
#include "direct_load.h"
#include "kernels.h"
#include "lds_layout.h"

#include <type_traits>
#include <utility>

namespace dash {

// compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>)
template <typename F, int... Is>
__device__ __forceinline__ void fstatic_for_impl(F&& f, std::integer_sequence<int, Is...>) {
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void fstatic_for(F&& f) {
    fstatic_for_impl(static_cast<F&&>(f), std::make_integer_sequence<int, N>{});
}


typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int BK = 16;             // K slab (32 measured slower: 125 against 128 TFLOP/s on a 128-block launch)
constexpr int MIN_WG = 2;          // workgroups per CU the compiler must leave room for (3 and 4 measured no better)
// workgroup shape per tile edge: WC x WC wavefronts, each computing a WT x WT part of the tile
//   TILE  64: 2 x 2 wavefronts of 32 x 32;  TILE 128: 2 x 2 wavefronts of 64 x 64 (256 threads);
//   (TILE 256 = 4 x 4 wavefronts of 64 x 64, 1024 threads, one workgroup per CU, also builds from this template: half the bytes
//   through the load path per flop; measured 2-3 % faster on launches of 128 blocks of 1024 and no faster on 32,
//   not used)
template <int TILE>
struct Cfg {
    static constexpr int WT = TILE == 64 ? 32 : 64;
    static constexpr int WC = TILE / WT;
    static constexpr int NW = WC * WC;
    static constexpr int NT = 64 * NW;
};
constexpr int NUM_XCD = 8;

// LDS layout of the operand slabs (lds_layout.h): chunks of 1 KB, one per wavefront-wide direct load; KC (k
// contiguous in memory) and RC (row contiguous) with their swizzles.
template <int TILE>
using Dma = layout::F32<TILE, BK, Cfg<TILE>::NW>;

// Byte offsets, inside the block and without the part that moves with the slab, of the cells one lane
// fetches: fixed for the whole tile, computed once, so that every load is "uniform base of the slab + per-lane
// offset".
template <int TILE, bool KC>
__device__ __forceinline__ void dma_offsets(int ld, int row0, int wave, int lane, unsigned (&off)[Dma<TILE>::NV]) {
#pragma unroll
    for (int u = 0; u < Dma<TILE>::NV; ++u) off[u] = Dma<TILE>::load_offset(KC, ld, row0, wave, lane, u);
}

// uniform byte offset of the slab starting at k0
template <bool KC>
__device__ __forceinline__ size_t slab_base(int ld, int k0) {
    return KC ? (size_t)k0 * 4 : (size_t)k0 * ld * 4;
}

// request one operand slab: global memory -> LDS.  `wave` must be uniform.
template <int TILE>
__device__ __forceinline__ void dma_load(const char* __restrict__ slab, const unsigned (&off)[Dma<TILE>::NV],
                                         float* __restrict__ dst, int wave) {
#pragma unroll
    for (int u = 0; u < Dma<TILE>::NV; ++u)
        direct_load16(slab, off[u], reinterpret_cast<char*>(dst) + Dma<TILE>::chunk(wave, u) * 1024);
}

// ---- LDS -> MFMA operand fragments for one chunk of 8 k --------------------------------
// For the MT sub-tiles of 32 rows of a wavefront, the first at r0: the four operand values a lane feeds to
// MFMA steps s = 0..3 of chunk c are the elements (r0 + 32 i + lane%32, 8c + 4*(lane/32) + s).  Per-lane float
// offsets are set up once; KC: one per chunk (the swizzle depends on it), the sub-tile adds a constant;
// RC: one per sub-tile (the swizzle flips bit 5 of the row), the chunk and the step add constants.
template <int TILE, bool KC, int MT>
struct Frag {
    typedef Dma<TILE> D;
    int fo[KC ? BK / 8 : MT];
    __device__ __forceinline__ void init(int r0, int lane) {
        if (KC) {
#pragma unroll
            for (int c = 0; c < BK / 8; ++c) fo[c] = D::frag_kc(r0, lane, c);
        } else {
#pragma unroll
            for (int i = 0; i < MT; ++i) fo[i] = D::frag_rc(r0, i, lane);
        }
    }
    __device__ __forceinline__ v4f read(const float* __restrict__ s, int i, int c) const {
        if (KC) return *reinterpret_cast<const v4f*>(s + fo[c] + i * D::KC_SUB);
        const float* p = s + fo[i] + 8 * c * TILE;
        v4f v;
        v[0] = p[0 * TILE];
        v[1] = p[1 * TILE];
        v[2] = p[2 * TILE];
        v[3] = p[3 * TILE];
        return v;
    }
};

// floats of LDS a workgroup of TILE needs: two stages of two operand slabs, or the epilogue strips
template <int TILE>
struct LdsNeed {
    static constexpr int STAGES = 2 * 2 * Dma<TILE>::SLAB;
    static constexpr int STRIPS = Cfg<TILE>::NW * 32 * (Cfg<TILE>::WT + 4);
    static constexpr int FLOATS = STAGES > STRIPS ? STAGES : STRIPS;
};

// One TILE x TILE output tile: workgroup `lid` of a part of a launch whose blocks start at blk_first.  Each
// wavefront owns WT x WT of the tile, i.e. MT x MT MFMA tiles of 32 x 32.  `lds` is the workgroup's LDS.
template <int TILE, bool TA, bool TB, bool RECT>
__device__ __forceinline__ void gemm_f32_tile(const GemmLaunch& g, int64_t lid, int64_t blk_first, float* lds) {
    constexpr int MT = Cfg<TILE>::WT / 32;
    constexpr bool A_KC = !TA;   // op(A)(i,k): k contiguous unless transposed
    constexpr bool B_KC = TB;    // op(B)(k,j): j contiguous unless transposed
    constexpr int NV = Dma<TILE>::NV;
    constexpr int SLAB = Dma<TILE>::SLAB;         // floats per operand slab; a stage is the A slab and the B slab
    constexpr int LDSF = LdsNeed<TILE>::FLOATS;

    // op(A) is Md x Kd, op(B) is Kd x Nd, C is Md x Nd (all equal to g.B unless a rectangular launch
    // sets g.M, g.N, g.K: ragged gradient blocks, paper Section 4.1 "rest" blocks)
    // (a separate instantiation: the square kernel keeps one dimension in registers)
    const int Md = RECT && g.M ? g.M : g.B, Nd = RECT && g.N ? g.N : Md, Kd = RECT && g.K ? g.K : Md;
    const int tiles = Md / TILE, tiles_n = Nd / TILE;
    const int T = g.sym ? tiles * (tiles + 1) / 2 : tiles * tiles_n;
    const int64_t blk = blk_first + lid / ((int64_t)g.nprob * T);
    const int r1 = (int)(lid % ((int64_t)g.nprob * T));
    const int pi = r1 / T;
    const int tile = r1 % T;
    int ti, tj;
    if (g.sym) {        // tiles of the upper triangle, row by row: (0,0..t-1), (1,1..t-1), ...
        int left = tile, len = tiles;
        ti = 0;
        while (left >= len) { left -= len; --len; ++ti; }
        tj = ti + left;
    } else {
        ti = tile / tiles_n;
        tj = tile % tiles_n;
    }
    const int row0 = ti * TILE;
    const int col0 = tj * TILE;

    const GemmProblem& P = g.prob[pi];
    const size_t boff = (size_t)blk * Md * Nd;          // C, D, C2
    const float* __restrict__ Ab = static_cast<const float*>(P.A) + (size_t)blk * Md * Kd;
    const float* __restrict__ Bb = static_cast<const float*>(P.B) + (size_t)blk * Kd * Nd;
    const int lda = TA ? Md : Kd, ldb = TB ? Kd : Nd;

    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = (wave / Cfg<TILE>::WC) * Cfg<TILE>::WT, wn = (wave % Cfg<TILE>::WC) * Cfg<TILE>::WT;

    v16f acc[MT][MT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < MT; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    unsigned offa[NV], offb[NV];
    dma_offsets<TILE, A_KC>(lda, row0, wave, lane, offa);
    dma_offsets<TILE, B_KC>(ldb, col0, wave, lane, offb);
    Frag<TILE, A_KC, MT> fra;
    Frag<TILE, B_KC, MT> frb;
    fra.init(wm, lane);
    frb.init(wn, lane);
    // uniform base addresses of the next slab to request, stepped: the K loop holds no address set-up
    const char* pa = reinterpret_cast<const char*>(Ab);
    const char* pb = reinterpret_cast<const char*>(Bb);
    const size_t stepa = slab_base<A_KC>(lda, BK), stepb = slab_base<B_KC>(ldb, BK);
    auto load_next = [&](float* stage) {
        dma_load<TILE>(pa, offa, stage, wave);
        dma_load<TILE>(pb, offb, stage + SLAB, wave);
        pa += stepa;
        pb += stepb;
    };
    // Fragments of chunk c live in register set c % 2; those of chunk c + 1 are requested before the MFMAs of
    // chunk c issue.
    constexpr int CH = BK / 8;
    v4f fa[2][MT], fb[2][MT];
    auto frags = [&](const float* sa, auto C) {
        constexpr int c = decltype(C)::value, b = c & 1;
#pragma unroll
        for (int i = 0; i < MT; ++i) fa[b][i] = fra.read(sa, i, c);
#pragma unroll
        for (int j = 0; j < MT; ++j) fb[b][j] = frb.read(sa + SLAB, j, c);
    };
    auto mfmas = [&](auto C) {
        constexpr int b = decltype(C)::value & 1;
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int j = 0; j < MT; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[b][i][s], fb[b][j][s], acc[i][j], 0, 0, 0);
    };
    // Two stages.  The barrier that opens slab h + 1 sits before the LAST chunk of slab h: by then a wavefront
    // holds all its fragments of slab h in registers, so the stage of slab h is free and slab h + 2 is requested
    // into it right after the barrier, and the first fragments of slab h + 1 are requested right after the
    // barrier while the MFMAs of the last chunk of slab h still run.  Before the barrier a wavefront waits until
    // its own loads of slab h + 1 have landed and its fragment reads are complete.
    const int KT = Kd / BK;
    load_next(lds);
    wait_vm_lgkm<0>();
    __builtin_amdgcn_s_barrier();
    if (1 < KT) load_next(lds + 2 * SLAB);
    frags(lds, std::integral_constant<int, 0>{});
    for (int h = 0; h < KT; ++h) {
        float* cur = lds + (h & 1) * 2 * SLAB;
        float* nxt = lds + ((h + 1) & 1) * 2 * SLAB;
        fstatic_for<CH - 1>([&](auto C) {
            frags(cur, std::integral_constant<int, decltype(C)::value + 1>{});
            mfmas(C);
        });
        if (h + 1 < KT) {
            wait_vm_lgkm<0>();
            __builtin_amdgcn_s_barrier();
            if (h + 2 < KT) load_next(cur);
            frags(nxt, std::integral_constant<int, 0>{});
        }
        mfmas(std::integral_constant<int, CH - 1>{});
    }
    __syncthreads();                    // every wavefront has left the last slab: LDS is free for the epilogue

    // ---- epilogue: C = mult * (alpha*acc + beta*D + gamma*I), staged through LDS ----
    // The MFMA leaves a lane with one column and scattered rows (register r of lane l holds row
    // 8*(r/4) + 4*(l/32) + r%4, column l%32 of its 32 x 32 tile): storing from there is 4 bytes per lane.
    // Instead every wavefront passes its accumulators, a strip of 32 rows x TILE/2 columns at a time,
    // through a private region of the (now free) operand buffers and comes back with row-contiguous
    // quads: D is read and C, C2 are written 16 bytes per lane.  Measured on 32 blocks of 1024: the
    // direct epilogue cost 8 % of the launch without D and 15 % with it.
    const float mult = P.mult ? P.mult[blk] : 1.f;
    const float alpha = P.alpha * mult, beta = P.beta * mult, gamma = P.gamma * mult;
    const float* __restrict__ Db = P.D ? P.D + boff : nullptr;
    float* __restrict__ Cb = P.C + boff;
    // optional second output C2 = a2 * C + g2 * I (Coupled-Newton: M' and C' = (1+1/p) I - M'/p at once)
    float* __restrict__ C2b = P.C2 ? P.C2 + boff : nullptr;
    const float a2 = P.a2, g2 = P.g2;
    // symmetric mode: an off-diagonal tile (ti < tj) is also written transposed to (tj, ti)
    const bool mirror = g.sym && ti != tj;
    constexpr int WT = Cfg<TILE>::WT;             // columns of a wavefront's strip
    constexpr int SP = WT + 4;                    // strip pitch in floats
    constexpr int QPR = WT / 4;                   // quads per strip row
    constexpr int RPI = 64 / QPR;                 // strip rows one pass of the wavefront covers
    static_assert(Cfg<TILE>::NW * 32 * SP <= LDSF, "strips must fit the LDS array");
    float* strip = lds + wave * 32 * SP;
    bool bad = false;
#pragma unroll
    for (int i = 0; i < MT; ++i) {
        // phase A: alpha * acc into the strip
#pragma unroll
        for (int j = 0; j < MT; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                strip[(8 * (r / 4) + 4 * (lane >> 5) + (r % 4)) * SP + 32 * j + (lane & 31)] = alpha * acc[i][j][r];
        __syncthreads();
        // phase B: row-contiguous quads
        const int rbase = row0 + wm + 32 * i, cbase = col0 + wn;
#pragma unroll 2
        for (int t = 0; t < 32 / RPI; ++t) {
            const int rl = lane / QPR + RPI * t, c = (lane % QPR) * 4;
            v4f v = *reinterpret_cast<const v4f*>(strip + rl * SP + c);
            const int row = rbase + rl, col = cbase + c;
            const size_t off = (size_t)row * Nd + col;
            if (Db) {
                const v4f d = *reinterpret_cast<const v4f*>(Db + off);
#pragma unroll
                for (int m = 0; m < 4; ++m) v[m] += beta * d[m];
            }
            v4f v2;
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                if (row == col + m) v[m] += gamma;
                bad |= !(fabsf(v[m]) <= 3.0e38f);
                v2[m] = a2 * v[m] + (row == col + m ? g2 : 0.f);
            }
            *reinterpret_cast<v4f*>(Cb + off) = v;
            if (C2b) *reinterpret_cast<v4f*>(C2b + off) = v2;
            if (mirror) *reinterpret_cast<v4f*>(strip + rl * SP + c) = v;      // final values for phase C
        }
        __syncthreads();
        // phase C (mirrored tiles only): a column of the strip is 32 consecutive elements of a row of the
        // transposed tile = one 128-byte line; eight lanes write it, four rows of the column each
        if (mirror) {
#pragma unroll 2
            for (int t = 0; t < WT / 8; ++t) {
                const int cl = (lane >> 3) + 8 * t, rl = 4 * (lane & 7);
                v4f v, v2;
#pragma unroll
                for (int m = 0; m < 4; ++m) {
                    v[m] = strip[(rl + m) * SP + cl];
                    v2[m] = a2 * v[m];                      // never on the diagonal
                }
                const size_t moff = (size_t)(cbase + cl) * Nd + rbase + rl;
                *reinterpret_cast<v4f*>(Cb + moff) = v;
                if (C2b) *reinterpret_cast<v4f*>(C2b + moff) = v2;
            }
            __syncthreads();
        }
    }
    if (g.nonfinite && pi == 0 && bad) g.nonfinite[blk] = 1;
}

// XCD-aware remap of a 1-D range of W workgroup ids: hardware hands consecutive ids to the 8 XCDs round-robin;
// the remapped id makes each XCD walk a contiguous range
__device__ __forceinline__ int64_t xcd_remap(int64_t bid, int64_t W) {
    const int64_t xcd = bid % NUM_XCD, local = bid / NUM_XCD;
    const int64_t per = W / NUM_XCD, rem = W % NUM_XCD;
    return xcd * per + (xcd < rem ? xcd : rem) + local;
}

// The launch: workgroups [0, g.w_main) compute TILE tiles of the first g.n_main blocks; when the launch is split
// (TILE 128, square products), workgroups from g.w_main on compute 64 tiles of the remaining blocks.  They have
// the same 256 threads and fit the same LDS, so they fill the CUs as the big tiles drain.
template <int TILE, bool TA, bool TB, bool RECT = false>
__global__ __launch_bounds__(Cfg<TILE>::NT, TILE == 256 ? 1 : MIN_WG) void gemm_f32_kernel(GemmLaunch g) {
    __shared__ __attribute__((aligned(1024))) float lds[LdsNeed<TILE>::FLOATS];
    const int64_t bid = blockIdx.x;
    if (TILE == 128 && !RECT) {
        static_assert(TILE != 128 || LdsNeed<64>::FLOATS <= LdsNeed<TILE>::FLOATS, "the 64 tile must fit");
        if (bid >= g.w_main) {
            gemm_f32_tile<64, TA, TB, false>(g, xcd_remap(bid - g.w_main, (int64_t)gridDim.x - g.w_main),
                                             g.blk0 + g.n_main, lds);
            return;
        }
        gemm_f32_tile<TILE, TA, TB, RECT>(g, xcd_remap(bid, g.w_main), g.blk0, lds);
    } else {
        gemm_f32_tile<TILE, TA, TB, RECT>(g, xcd_remap(bid, gridDim.x), g.blk0, lds);
    }
}

// The factor accumulation: product 0 of every block is A B^T (G G^T), product 1 is A^T B (G^T G) -- two memory
// orders, two instances of the tile function, one launch, so that the 2 x 36 tiles of a block fill the chip
// together (each product alone is half a round of workgroups on the benchmark's 16 gradient blocks).
template <int TILE>
__device__ __forceinline__ void gemm_f32_pair_tile(const GemmLaunch& g, int64_t lid, int64_t blk_first, float* lds) {
    const int tiles = g.B / TILE;
    const int T = g.sym ? tiles * (tiles + 1) / 2 : tiles * tiles;
    const int pi = (int)(lid % ((int64_t)2 * T)) / T;         // as the tile function will find it
    if (pi == 0) gemm_f32_tile<TILE, false, true, false>(g, lid, blk_first, lds);
    else gemm_f32_tile<TILE, true, false, false>(g, lid, blk_first, lds);
}

template <int TILE>
__global__ __launch_bounds__(Cfg<TILE>::NT, MIN_WG) void gemm_f32_pair_kernel(GemmLaunch g) {
    __shared__ __attribute__((aligned(1024))) float lds[LdsNeed<TILE>::FLOATS];
    const int64_t bid = blockIdx.x;
    if (TILE == 128) {
        if (bid >= g.w_main) {
            gemm_f32_pair_tile<64>(g, xcd_remap(bid - g.w_main, (int64_t)gridDim.x - g.w_main), g.blk0 + g.n_main, lds);
            return;
        }
        gemm_f32_pair_tile<TILE>(g, xcd_remap(bid, g.w_main), g.blk0, lds);
    } else {
        gemm_f32_pair_tile<TILE>(g, xcd_remap(bid, gridDim.x), g.blk0, lds);
    }
}

// the one two-product launch with different memory orders: (A B^T, A^T B) on square fp32 blocks
static bool gemm_is_pair(const GemmLaunch& g) {
    return g.nprob == 2 && g.half == HALF_NONE && !g.M && !g.N && !g.K && !g.prob[0].transA && g.prob[0].transB &&
           g.prob[1].transA && !g.prob[1].transB;
}

// workgroups of nblocks blocks computed with TILE tiles
template <int TILE>
static int64_t tile_count(const GemmLaunch& g, int64_t nblocks) {
    const int64_t tiles = (g.M ? g.M : g.B) / TILE, tiles_n = (g.N ? g.N : g.B) / TILE;
    return nblocks * g.nprob * (g.sym ? tiles * (tiles + 1) / 2 : tiles * tiles_n);
}

// n_main blocks with TILE tiles; the remaining blocks (TILE 128 only) with 64 tiles in the same launch
template <int TILE>
static hipError_t launch_tile(const GemmLaunch& g0, int64_t n_main, hipStream_t stream) {
    GemmLaunch g = g0;
    g.n_main = n_main;
    g.w_main = tile_count<TILE>(g, n_main);
    const int64_t W = g.w_main + (n_main < g.nblocks ? tile_count<64>(g, g.nblocks - n_main) : 0);
    if (W <= 0) return hipSuccess;
    if (W > 0x7fffffffLL) return hipErrorInvalidValue;
    const int ta = g.prob[0].transA, tb = g.prob[0].transB;
    dim3 grid((unsigned)W), block(Cfg<TILE>::NT);
    if (gemm_is_pair(g)) {
        hipLaunchKernelGGL((gemm_f32_pair_kernel<TILE>), grid, block, 0, stream, g);
        return hipGetLastError();
    }
    // otherwise both products of a launch use the same transpose flags (one kernel instance)
    if (g.M || g.N || g.K) {
        if (!ta && !tb) hipLaunchKernelGGL((gemm_f32_kernel<TILE, false, false, true>), grid, block, 0, stream, g);
        else if (!ta && tb) hipLaunchKernelGGL((gemm_f32_kernel<TILE, false, true, true>), grid, block, 0, stream, g);
        else if (ta && !tb) hipLaunchKernelGGL((gemm_f32_kernel<TILE, true, false, true>), grid, block, 0, stream, g);
        else hipLaunchKernelGGL((gemm_f32_kernel<TILE, true, true, true>), grid, block, 0, stream, g);
        return hipGetLastError();
    }
    if (!ta && !tb) hipLaunchKernelGGL((gemm_f32_kernel<TILE, false, false>), grid, block, 0, stream, g);
    else if (!ta && tb) hipLaunchKernelGGL((gemm_f32_kernel<TILE, false, true>), grid, block, 0, stream, g);
    else if (ta && !tb) hipLaunchKernelGGL((gemm_f32_kernel<TILE, true, false>), grid, block, 0, stream, g);
    else hipLaunchKernelGGL((gemm_f32_kernel<TILE, true, true>), grid, block, 0, stream, g);
    return hipGetLastError();
}

hipError_t launch_gemm(const GemmLaunch& g, hipStream_t stream) {
    if (g.nprob < 1 || g.nprob > 2 || g.B <= 0 || g.B % 64) return hipErrorInvalidValue;
    if (g.M % 64 || g.N % 64 || g.K % 64 || g.M < 0 || g.N < 0 || g.K < 0) return hipErrorInvalidValue;
    const bool rect = g.M || g.N || g.K;
    if (rect && g.half != HALF_NONE) return hipErrorInvalidValue;              // rectangular: fp32 only
    if (g.sym && (g.M ? g.M : g.B) != (g.N ? g.N : g.B)) return hipErrorInvalidValue;   // mirroring needs a square output
    if (g.nprob == 2 && !gemm_is_pair(g) &&
        (g.prob[0].transA != g.prob[1].transA || g.prob[0].transB != g.prob[1].transB))
        return hipErrorInvalidValue;
    if (g.half != HALF_NONE) return launch_gemm_half(g, stream);
    if (gemm_tile_edge(g) != 128) return launch_tile<64>(g, g.nblocks, stream);
    // whole rounds with 128 tiles; the last blocks, if any, with 64 tiles behind them in the same launch (same
    // result bit for bit: an output element is accumulated over k in the same order whatever the tile)
    return launch_tile<128>(g, gemm_split_blocks(g), stream);
}

// 128-wide tiles when they still give the chip enough workgroups, else 64-wide.  A launch of fewer 128-tile
// workgroups than fit the chip at once (1024) is resident as a whole, and it takes as long as the CU with the most
// workgroups: when the workgroups fill less than 86 % of whole layers of one per CU (a Clenshaw product on 64
// blocks of 512 is 640 workgroups: 2.5 per CU), 64 tiles, four times as many and dealt out as slots free up,
// balance better than the bigger tile is faster (measured 10-16 % on such launches).
int gemm_tile_edge(const GemmLaunch& g) {
    const int Md = g.M ? g.M : g.B, Nd = g.N ? g.N : g.B, Kd = g.K ? g.K : g.B;
    (void)Kd;                                     // the K loop only needs K % 16 == 0
    const bool big = Md % 128 == 0 && Nd % 128 == 0 &&
                     g.nblocks * g.nprob * (int64_t)(Md / 128) * (Nd / 128) >= 256;
    if (!big) return 64;
    const int64_t tm = Md / 128, tn = Nd / 128;
    const int64_t w = g.nblocks * g.nprob * (g.sym ? tm * (tm + 1) / 2 : tm * tn);     // 128-tile workgroups
    if (g.half == HALF_NONE && w < 1024) {     // (fp32 launches: the 16-bit kernel has other residency)
        const int64_t layers = (w + 255) / 256;
        if (100 * w < 86 * 256 * layers) return 64;
    }
    return 128;
}

// A launch of 128 tiles runs in rounds of RESIDENT workgroups (four per CU).  When the last round would be
// less than half full - every CU then ends with one lonely workgroup, or none - the blocks that fill whole
// rounds keep the 128 tiles and the remaining blocks are computed with 64 tiles, which spread over all CUs.
// Returns the number of blocks of the first part (nblocks: no split).
int64_t gemm_split_blocks(const GemmLaunch& g) {
    constexpr int64_t RESIDENT = 4 * 256;
    if (g.half != HALF_NONE || g.M || g.N || g.K || gemm_tile_edge(g) != 128) return g.nblocks;
    const int64_t tm = (g.M ? g.M : g.B) / 128, tn = (g.N ? g.N : g.B) / 128;
    const int64_t per_block = g.nprob * (g.sym ? tm * (tm + 1) / 2 : tm * tn);
    const int64_t W = g.nblocks * per_block;
    const int64_t full = W / RESIDENT, rem = W % RESIDENT;
    if (full < 1 || rem == 0 || rem > RESIDENT / 2) return g.nblocks;
    const int64_t na = full * RESIDENT / per_block;
    return na >= 1 && na < g.nblocks ? na : g.nblocks;
}

// fraction of the B x B output tiles a launch computes (1, or (t+1)/(2t) in symmetric mode, t = tiles per edge)
double gemm_tile_fraction(const GemmLaunch& g) {
    if (!g.sym) return 1.0;
    const int Md = g.M ? g.M : g.B;
    if (g.half != HALF_NONE) {
        const int edge = gemm_half_tile_edge(g);
        const int t = Md / edge;
        const double f = (double)(t + 1) / (2.0 * t);
        const int64_t na = gemm_half_split_blocks(g);      // blocks computed with the launch's own tile; the rest with 128
        if (na == g.nblocks) return f;
        const int t128 = Md / 128;
        const double f128 = (double)(t128 + 1) / (2.0 * t128);
        return (f * (double)na + f128 * (double)(g.nblocks - na)) / (double)g.nblocks;
    }
    const int t = Md / gemm_tile_edge(g);
    const double f = (double)(t + 1) / (2.0 * t);
    const int64_t na = gemm_split_blocks(g);
    if (na == g.nblocks) return f;
    const int t64 = Md / 64;
    const double f64 = (double)(t64 + 1) / (2.0 * t64);
    return (f * (double)na + f64 * (double)(g.nblocks - na)) / (double)g.nblocks;
}

}  // namespace dash
