// Batched B x B x B matmul with 16-bit operands (bf16 or fp16) and fp32 accumulation, for gfx950.
//
// Mixed-precision form of the same product as gemm.hip (paper Appendix A.3: iterates are
// kept in fp32, the operands of each matmul are rounded to half precision, accumulation
// is fp32; the paper uses fp16, the bf16 form is the one its Section 5 reports unstable for
// Newton-DB).  Operands arrive already rounded: the epilogue of the product (or the
// elementwise kernel) that produced an iterate writes a 16-bit copy next to, or instead of,
// the fp32 value, so no separate cast pass exists.
//     acc = op(A_b) op(B_b)             (v_mfma_f32_32x32x16_bf16 / v_mfma_f32_32x32x16_f16)
//     v   = mult_b * (alpha * acc + beta * D_b + gamma * I)     (fp32)
//     C_b = v (fp32, optional),  Ch_b = half(v) (optional),  C2h_b = half(a2 v + g2 I) (optional)
//
// Same decomposition as the fp32 kernel: TILE x TILE per workgroup (2 x 2 wavefronts, or 4 x 4
// for the 256 tile), K slabs of 64 double-buffered in LDS, LDS-staged epilogue, XCD-aware 1-D grid.
// Operand slabs go from global memory straight into LDS (global_load_lds_dwordx4: a wavefront-wide
// load fills 1 KB of LDS in lane order, the source address of every lane is free), one slab ahead
// of the MFMAs, so no registers and no LDS store instructions are spent on staging.  An MFMA
// operand wants per lane eight consecutive k of one row:
//   KC  [row][k]  k contiguous in global memory: LDS holds rows of 64 k (128 bytes, cells of 16
//       bytes swizzled inside the row), one 16-byte LDS read per MFMA operand;
//   KR  [k][row]  row contiguous in global memory: LDS holds the k-lines as they are in memory
//       (cells swizzled inside the line) and the operand is assembled by two transposing reads
//       (ds_read_b64_tr_b16: sixteen lanes read a 4 x 16 patch of 16-bit values and each gets
//       one column of it).
#include "direct_load.h"
#include "kernels.h"
#include "lds_layout.h"

#include <type_traits>
#include <utility>

namespace dash {

constexpr int64_t H256_MIN_WORKGROUPS = 128;   // workgroups a launch must have for the 256 tile (measured: 64, 96, 160 and 256 all lose)

// compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>).  The accumulator
// array must only ever be indexed by constants, or the compiler moves it to scratch memory; a pragma
// does not guarantee that once the body is long.
template <typename F, int... Is>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, Is...>) {
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    static_for_impl(static_cast<F&&>(f), std::make_integer_sequence<int, N>{});
}

typedef float v16f __attribute__((ext_vector_type(16)));
typedef unsigned short u16;      // a 16-bit operand element while it is only being moved
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef u16 v4s __attribute__((ext_vector_type(4)));

// the two 16-bit operand formats: conversion from fp32 (round to nearest even) and the MFMA
struct Bf16 {
    static constexpr float LO_SCALE = 1.f;      // bf16 has the exponent range of fp32: low planes need no scaling
    typedef __bf16 v8 __attribute__((ext_vector_type(8)));
    static __device__ __forceinline__ u16 from_float(float v) {
        union { __bf16 h; u16 u; } x; x.h = (__bf16)v; return x.u;
    }
    static __device__ __forceinline__ float to_float(u16 u) {
        union { __bf16 h; u16 u; } x; x.u = u; return (float)x.h;
    }
    static __device__ __forceinline__ v16f mfma(v4u a, v4u b, v16f c) {
        union { v4u u; v8 h; } x, y; x.u = a; y.u = b;
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(x.h, y.h, c, 0, 0, 0);
    }
};
struct Fp16 {
    // two-plane mode: the low plane is 2^-11 of the value or less and would go subnormal in fp16 for |x| < 0.125;
    // it is stored times 2^11, and the sum of the two segments that read a low plane is scaled back once
    static constexpr float LO_SCALE = 2048.f;
    typedef _Float16 v8 __attribute__((ext_vector_type(8)));
    static __device__ __forceinline__ u16 from_float(float v) {
        union { _Float16 h; u16 u; } x; x.h = (_Float16)v; return x.u;
    }
    static __device__ __forceinline__ float to_float(u16 u) {
        union { _Float16 h; u16 u; } x; x.u = u; return (float)x.h;
    }
    static __device__ __forceinline__ v16f mfma(v4u a, v4u b, v16f c) {
        union { v4u u; v8 h; } x, y; x.u = a; y.u = b;
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(x.h, y.h, c, 0, 0, 0);
    }
};

namespace {

// workgroup shape per tile edge: WC x WC wavefronts, each computing a WT x WT part of the tile; K slabs of
// HBK elements in a ring of NS LDS stages (NS - 1 slabs are in flight while one is multiplied)
//   TILE  64: 2 x 2 wavefronts of 32 x 32   (256 threads), slabs of 64, 2 stages
//   TILE 128: 2 x 2 wavefronts of 64 x 64   (256 threads, two workgroups per CU), slabs of 64, 2 stages
//   TILE 256: 4 x 4 wavefronts of 64 x 64  (1024 threads, one workgroup per CU: the same four wavefronts
//             per SIMD as two 128 tiles, but every operand panel fetched from L2 serves twice the flops),
//             slabs of 64, 2 stages (slabs of 32 in rings of 3 to 5 stages build as well and measured slower)
template <int TILE>
struct HCfg {
    static constexpr int WT = TILE == 64 ? 32 : 64;
    static constexpr int WC = TILE / WT;
    static constexpr int NT = 64 * WC * WC;
    static constexpr int OCC = TILE == 256 ? 1 : 2;        // workgroups per CU the kernel is built for
    static constexpr int HBK = 64;                          // K slab (slabs of 32 in rings of 3 to 5 stages measured slower)
    static constexpr int NS = 2;                            // stages of the ring
};
constexpr int HNUM_XCD = 8;

// LDS layout of the operand slabs (lds_layout.h): chunks of 1 KB, one per wavefront-wide direct load; KC (k
// contiguous in memory) and KR (row contiguous) with their swizzles.
template <int TILE>
using HDma = layout::Half<TILE, HCfg<TILE>::HBK, HCfg<TILE>::NT / 64>;

// Byte offsets, inside the block and without the part that moves with the slab, of the cells one lane
// fetches: fixed for the whole tile, computed once, so that every load is "uniform base of the slab + per-lane
// offset".
template <int TILE, bool KC>
__device__ __forceinline__ void hdma_offsets(int ld, int row0, int wave, int lane, unsigned (&off)[HDma<TILE>::NV]) {
#pragma unroll
    for (int u = 0; u < HDma<TILE>::NV; ++u) off[u] = HDma<TILE>::load_offset(KC, ld, row0, wave, lane, u);
}

// uniform byte offset of slab k0 inside the block
template <bool KC>
__device__ __forceinline__ size_t hslab_base(int ld, int k0) {
    return KC ? (size_t)k0 * 2 : (size_t)k0 * ld * 2;
}

// request one operand slab: global memory -> LDS, no registers in between.  `wave` must be uniform.
template <int TILE>
__device__ __forceinline__ void hdma_load(const char* __restrict__ slab, const unsigned (&off)[HDma<TILE>::NV],
                                          char* __restrict__ dst, int wave) {
    typedef HDma<TILE> D;
#pragma unroll
    for (int u = 0; u < D::NV; ++u) direct_load16(slab, off[u], dst + D::chunk(wave, u) * 1024);
}

// Per-lane LDS byte offsets of the operand fragments of a wavefront's MT sub-tiles of 32 rows, the first at
// r0.  KC: one offset per MFMA step (the swizzle depends on the step), the sub-tile adds an immediate; KR: one
// offset per sub-tile (the swizzle depends on it), the step adds an immediate.
template <int TILE, bool KC, int MT>
struct HFrag {
    typedef HDma<TILE> D;
    int base[KC ? D::STEPS : MT];
    __device__ __forceinline__ void init(int r0, int lane) {
        if (KC) {
#pragma unroll
            for (int st = 0; st < D::STEPS; ++st) base[st] = D::frag_kc(r0, lane, st);
        } else {
#pragma unroll
            for (int i = 0; i < MT; ++i) base[i] = D::frag_kr(r0, i, lane);
        }
    }
    __device__ __forceinline__ v4u read(const char* __restrict__ s, int i, int st) const {
        if (KC) return *reinterpret_cast<const v4u*>(s + base[st] + i * D::KC_SUB);
        typedef short v4h __attribute__((ext_vector_type(4)));
        typedef v4h __attribute__((address_space(3))) * lptr;
        const char* p = s + base[i] + st * D::KR_STEP;
        union { v4h h[2]; v4u u; } x;
        x.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lptr)(p));
        x.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lptr)(p + D::KR_HALF));
        return x.u;
    }
};

template <typename H, int TILE, bool TA, bool TB>
__global__ __launch_bounds__(HCfg<TILE>::NT, HCfg<TILE>::OCC) void gemm_half_kernel(GemmLaunch g) {
    constexpr int MT = HCfg<TILE>::WT / 32;
    constexpr bool A_KC = !TA;
    constexpr bool B_KC = TB;
    constexpr int NV = HDma<TILE>::NV;
    constexpr int SLAB = HDma<TILE>::SLAB;
    constexpr int HBK = HCfg<TILE>::HBK;
    constexpr int NS = HCfg<TILE>::NS;
    static_assert(NS >= 2 && NS <= 5, "two to five stages");

    // one object per stage: the compiler then knows that fragment reads of one stage cannot touch the others,
    // into which later slabs are in flight, and does not wait for those loads before the reads
    __shared__ __attribute__((aligned(1024))) char stage0[2 * SLAB];
    __shared__ __attribute__((aligned(1024))) char stage1[2 * SLAB];
    __shared__ __attribute__((aligned(1024))) char stage2[NS > 2 ? 2 * SLAB : 1024];
    __shared__ __attribute__((aligned(1024))) char stage3[NS > 3 ? 2 * SLAB : 1024];
    __shared__ __attribute__((aligned(1024))) char stage4[NS > 4 ? 2 * SLAB : 1024];
    auto stage = [&](auto S) -> char* {
        constexpr int st = decltype(S)::value;
        if constexpr (st == 0) return stage0;
        else if constexpr (st == 1) return stage1;
        else if constexpr (st == 2) return stage2;
        else if constexpr (st == 3) return stage3;
        else return stage4;
    };

    const int64_t W = gridDim.x;
    const int64_t bid = blockIdx.x;
    const int64_t xcd = bid % HNUM_XCD, local = bid / HNUM_XCD;
    const int64_t per = W / HNUM_XCD, rem = W % HNUM_XCD;
    const int64_t lid = xcd * per + (xcd < rem ? xcd : rem) + local;

    const int B = g.B;
    const int tiles = B / TILE;
    const int T = g.sym ? tiles * (tiles + 1) / 2 : tiles * tiles;
    const int64_t blk = g.blk0 + lid / ((int64_t)g.nprob * T);
    const int r1 = (int)(lid % ((int64_t)g.nprob * T));
    const int pi = r1 / T;
    const int tile = r1 % T;
    int ti, tj;
    if (g.sym) {        // tiles of the upper triangle, row by row
        int left = tile, len = tiles;
        ti = 0;
        while (left >= len) { left -= len; --len; ++ti; }
        tj = ti + left;
    } else {
        ti = tile / tiles;
        tj = tile % tiles;
    }
    const int row0 = ti * TILE;
    const int col0 = tj * TILE;

    const GemmProblem& P = g.prob[pi];
    const size_t boff = (size_t)blk * B * B;
    // Split-operand mode (A2, B2 given): every operand is the sum of a high and a low 16-bit plane
    // (x ~ hi + lo, hi = round(x), lo = round(x - hi)) and the product is A_lo B_hi + A_hi B_lo + A_hi B_hi,
    // i.e. one product whose K runs over three segments with different plane pairs (lo*lo is dropped).
    // Three-plane mode (A3, B3 given as well, x ~ hi + mid + lo): the six plane products of weight 2^-16 and
    // above, A_lo B_hi + A_hi B_lo + A_mid B_mid + A_mid B_hi + A_hi B_mid + A_hi B_hi.
    // Segments are numbered so that every mode runs a tail of the same list, small terms first:
    //   0: A3 B   1: A B3   2: A2 B2   3: A2 B   4: A B2   5: A B
    const int nseg = P.A3 ? 6 : P.A2 ? 3 : 1;
    // (the plane pointers are fetched from the launch arguments when a segment begins: six more pointers held
    // in scalar registers through the K loop would not fit)
    auto seg_a = [&](int sg) {
        const void* q = sg == 0 ? P.A3 : (sg == 2 || sg == 3) ? P.A2 : P.A;
        return static_cast<const char*>(q) + boff * sizeof(u16);
    };
    auto seg_b = [&](int sg) {
        const void* q = sg == 1 ? P.B3 : (sg == 2 || sg == 4) ? P.B2 : P.B;
        return static_cast<const char*>(q) + boff * sizeof(u16);
    };

    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = (wave / HCfg<TILE>::WC) * HCfg<TILE>::WT, wn = (wave % HCfg<TILE>::WC) * HCfg<TILE>::WT;

    v16f acc[MT][MT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < MT; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int KS = B / HBK;             // slabs per segment
    const int KT = nseg * KS;           // slabs in all
    const int scale_at = nseg == 3 ? 2 * KS : -1;     // first slab of the high-high segment of a two-plane product
    unsigned offa[NV], offb[NV];
    hdma_offsets<TILE, A_KC>(B, row0, wave, lane, offa);
    hdma_offsets<TILE, B_KC>(B, col0, wave, lane, offb);
    HFrag<TILE, A_KC, MT> fra;
    HFrag<TILE, B_KC, MT> frb;
    fra.init(wm, lane);
    frb.init(wn, lane);
    // The slabs are requested in order, segment after segment (the small terms are summed first; a plain
    // product is the last segment alone).  The uniform base
    // addresses of the next slab are carried along and stepped, so the K loop holds no address set-up.
    const size_t stepa = hslab_base<A_KC>(B, HBK), stepb = hslab_base<B_KC>(B, HBK);
    int seg_next = 6 - nseg, ks_next = 0;
    const char* pa = seg_a(seg_next);
    const char* pb = seg_b(seg_next);
    auto load_next = [&](char* dst) {
        hdma_load<TILE>(pa, offa, dst, wave);
        hdma_load<TILE>(pb, offb, dst + SLAB, wave);
        if (++ks_next < KS) {
            pa += stepa;
            pb += stepb;
        } else {
            ks_next = 0;
            ++seg_next;
            pa = seg_a(seg_next);
            pb = seg_b(seg_next);
        }
    };
    // Fragments of MFMA step st live in register set st % 2; those of step st + 1 are requested before the MFMAs
    // of step st issue.
    constexpr int STEPS = HBK / 16;
    v4u fa[2][MT], fb[2][MT];
    auto frags = [&](const char* sa, auto ST) {
        constexpr int st = decltype(ST)::value, b = st & 1;
#pragma unroll
        for (int i = 0; i < MT; ++i) fa[b][i] = fra.read(sa, i, st);
#pragma unroll
        for (int j = 0; j < MT; ++j) fb[b][j] = frb.read(sa + SLAB, j, st);
    };
    auto mfmas = [&](auto ST) {
        constexpr int b = decltype(ST)::value & 1;
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int j = 0; j < MT; ++j)
                acc[i][j] = H::mfma(fa[b][i], fb[b][j], acc[i][j]);
    };
    // Ring of NS stages.  The barrier that opens slab h + 1 sits before the LAST MFMA step of slab h: by then
    // a wavefront holds all its fragments of slab h in registers, so (a) the stage of slab h is free and slab
    // h + NS is requested into it right after the barrier, (b) the first fragments of slab h + 1 are
    // requested right after the barrier and the MFMAs of the last step of slab h cover the moment when all
    // wavefronts of the workgroup hit the LDS together.  Before the barrier a wavefront waits until its own
    // loads of slab h + 1 have landed (those of later slabs may still be under way: the counter retires loads
    // in order) and its fragment reads are complete.  The ring is unrolled so that the stage of a slab is a
    // compile-time constant.
    constexpr int LATER = 2 * NV * (NS - 2);        // loads of one wavefront that may stay in flight at a barrier
    static_for<NS - 1>([&](auto S) {
        if (decltype(S)::value < KT) load_next(stage(S));
    });
    if (NS - 2 < KT) wait_vm_lgkm<LATER>();
    else wait_vm_lgkm<0>();
    __builtin_amdgcn_s_barrier();
    if (NS - 1 < KT) load_next(stage(std::integral_constant<int, NS - 1>{}));
    frags(stage0, std::integral_constant<int, 0>{});
    for (int h0 = 0; h0 < KT; h0 += NS) {
        static_for<NS>([&](auto S) {
            constexpr int sg = decltype(S)::value;
            const int h = h0 + sg;
            if (h < KT) {
                if (H::LO_SCALE != 1.f && h == scale_at) {       // the two low-plane segments are done: undo their scale
#pragma unroll
                    for (int i = 0; i < MT; ++i)
#pragma unroll
                        for (int j = 0; j < MT; ++j)
#pragma unroll
                            for (int r = 0; r < 16; ++r) acc[i][j][r] *= 1.f / H::LO_SCALE;
                }
                const char* cur = stage(S);
                static_for<STEPS - 1>([&](auto ST) {
                    frags(cur, std::integral_constant<int, decltype(ST)::value + 1>{});
                    mfmas(ST);
                });
                if (h + 1 < KT) {
                    if (h + NS - 1 < KT) wait_vm_lgkm<LATER>();
                    else wait_vm_lgkm<0>();
                    __builtin_amdgcn_s_barrier();
                    if (h + NS < KT) load_next(stage(S));
                    frags(stage(std::integral_constant<int, (sg + 1) % NS>{}), std::integral_constant<int, 0>{});
                }
                mfmas(std::integral_constant<int, STEPS - 1>{});
            }
        });
    }
    __syncthreads();                    // every wavefront has left the last slab: LDS is free for the epilogue

    // ---- epilogue, staged through LDS (free after the last barrier of the main loop) ----
    // The MFMA leaves a lane with one column and scattered rows; storing from there means 4-byte (or
    // 2-byte) stores and a fully unrolled epilogue whose code no longer fits the instruction cache.
    // Instead every wavefront passes its accumulators, one strip of 16 rows x WT columns at a time,
    // through a private LDS region and comes back with row-contiguous quads: 16-byte loads of D,
    // 16-byte stores of fp32 outputs, 8-byte stores of 16-bit outputs, in a compact loop.
    const float mult = P.mult ? P.mult[blk] : 1.f;
    const float alpha = P.alpha * mult, beta = P.beta * mult, gamma = P.gamma * mult;
    const float* __restrict__ Db = P.D ? P.D + boff : nullptr;
    float* __restrict__ Cb = P.C ? P.C + boff : nullptr;
    u16* __restrict__ Hb = P.Ch ? static_cast<u16*>(P.Ch) + boff : nullptr;
    u16* __restrict__ H2b = P.C2h ? static_cast<u16*>(P.C2h) + boff : nullptr;
    u16* __restrict__ H2lb = P.C2l ? static_cast<u16*>(P.C2l) + boff : nullptr;     // planes of the second output
    u16* __restrict__ H2l2b = P.C2l2 ? static_cast<u16*>(P.C2l2) + boff : nullptr;  // (with Cl2, as for the first output)
    u16* __restrict__ Lb = P.Cl ? static_cast<u16*>(P.Cl) + boff : nullptr;    // low plane of the result
    u16* __restrict__ L2b = P.Cl2 ? static_cast<u16*>(P.Cl2) + boff : nullptr; // third plane (with Lb only)
    const float lo_scale = P.Cl2 ? 1.f : H::LO_SCALE;     // two-plane results: the low plane is stored scaled
    const float a2 = P.a2, g2 = P.g2;
    // symmetric mode: an off-diagonal tile is also written transposed
    const bool mirror = g.sym && ti != tj;
    constexpr int WT = HCfg<TILE>::WT;            // columns of a wavefront's strip
    constexpr int QPR = WT / 4;                   // quads per strip row
    constexpr int RPI = 64 / QPR;                 // strip rows one pass of the wavefront covers
    constexpr int SPS = 2 * SLAB / (16 * WT * 4);     // strips one stage holds
    static_assert(SPS >= 1 && (HCfg<TILE>::NT / 64 + SPS - 1) / SPS <= 2, "strips must fit the first two stages");
    // strip rows are not padded; rows whose bit 2 is set swap their column halves instead, which keeps the two
    // rows (r, r + 4) that one MFMA register spreads over the lane halves in different banks
    float* strip = reinterpret_cast<float*>(wave < SPS ? stage0 : stage1) + (wave % SPS) * 16 * WT;
    auto swz = [](int row) { return (WT / 2) * ((row >> 2) & 1); };
    bool bad = false;
    static_for<2 * MT>([&](auto IH) {
        constexpr int i = decltype(IH)::value / 2, hs = decltype(IH)::value % 2;     // sub-tile, half of it
        // phase A: alpha * acc into the strip, element (8 (q%2) + 4 (lane/32) + m, 32 j + lane%32), q = r/4, m = r%4
        static_for<MT>([&](auto J) {
            constexpr int j = decltype(J)::value;
#pragma unroll
            for (int r8 = 0; r8 < 8; ++r8) {
                const int rl = 8 * (r8 / 4) + 4 * (lane >> 5) + (r8 % 4);
                strip[rl * WT + ((32 * j + (lane & 31)) ^ swz(rl))] = alpha * acc[i][j][8 * hs + r8];
            }
        });
        // The strip belongs to this wavefront alone, and the LDS executes the accesses of one wavefront in the
        // order they were issued: no barrier between the phases, the compiler only has to keep that order.
        __builtin_amdgcn_wave_barrier();
        // phase B: row-contiguous quads.  Strips that the diagonal does not cross (the common case) skip all
        // diagonal handling; outputs that were not asked for cost nothing.
        const int rbase = row0 + wm + 32 * i + 16 * hs, cbase = col0 + wn;
        auto quads = [&](auto DIAG) {
            constexpr bool diag = decltype(DIAG)::value;
#pragma unroll 1
            for (int t = 0; t < 16 / RPI; ++t) {
                const int rl = lane / QPR + RPI * t, c = (lane % QPR) * 4;
                float* sp = strip + rl * WT + (c ^ swz(rl));
                v4f v = *reinterpret_cast<const v4f*>(sp);
                const int row = rbase + rl, col = cbase + c;
                const size_t off = (size_t)row * B + col;
                if (Db) {
                    const v4f d = *reinterpret_cast<const v4f*>(Db + off);
#pragma unroll
                    for (int m = 0; m < 4; ++m) v[m] += beta * d[m];
                }
#pragma unroll
                for (int m = 0; m < 4; ++m) {
                    if (diag && row == col + m) v[m] += gamma;
                    bad |= !(fabsf(v[m]) <= 3.0e38f);
                }
                if (Cb) *reinterpret_cast<v4f*>(Cb + off) = v;
                if (Hb || Lb) {
                    v4s h;
#pragma unroll
                    for (int m = 0; m < 4; ++m) h[m] = H::from_float(v[m]);
                    if (Hb) *reinterpret_cast<v4s*>(Hb + off) = h;
                    if (Lb) {                     // split modes only: the plain product pays nothing for them
                        v4s lo;
                        float rest[4];
#pragma unroll
                        for (int m = 0; m < 4; ++m) {
                            rest[m] = v[m] - H::to_float(h[m]);
                            lo[m] = H::from_float(rest[m] * lo_scale);
                        }
                        *reinterpret_cast<v4s*>(Lb + off) = lo;
                        if (L2b) {
                            v4s lo2;
#pragma unroll
                            for (int m = 0; m < 4; ++m) lo2[m] = H::from_float(rest[m] - H::to_float(lo[m]));
                            *reinterpret_cast<v4s*>(L2b + off) = lo2;
                        }
                    }
                }
                if (H2b) {
                    v4s h2;
                    float w[4];
#pragma unroll
                    for (int m = 0; m < 4; ++m) {
                        w[m] = a2 * v[m] + (diag && row == col + m ? g2 : 0.f);
                        h2[m] = H::from_float(w[m]);
                    }
                    *reinterpret_cast<v4s*>(H2b + off) = h2;
                    if (H2lb) {
                        v4s lo, lo2;
#pragma unroll
                        for (int m = 0; m < 4; ++m) {
                            const float rest = w[m] - H::to_float(h2[m]);
                            lo[m] = H::from_float(rest * lo_scale);
                            lo2[m] = H::from_float(rest - H::to_float(lo[m]));    // (three planes: lo_scale is 1)
                        }
                        *reinterpret_cast<v4s*>(H2lb + off) = lo;
                        if (H2l2b) *reinterpret_cast<v4s*>(H2l2b + off) = lo2;
                    }
                }
                if (mirror) *reinterpret_cast<v4f*>(sp) = v;       // final values for phase C
            }
        };
        if (rbase + 16 > cbase && rbase < cbase + WT) quads(std::true_type{});
        else quads(std::false_type{});
        __builtin_amdgcn_wave_barrier();
        // phase C (mirrored tiles only, never on the diagonal): back in the MFMA layout a lane holds four
        // consecutive rows of one column = four consecutive elements of a row of the transposed tile
        if (mirror) {
#pragma unroll 1
            for (int jq = 0; jq < MT * 2; ++jq) {
                const int j = jq >> 1, q = jq & 1;
                const int rl = 8 * q + 4 * (lane >> 5), cl = 32 * j + (lane & 31);
                const int row = rbase + rl, col = cbase + cl;
                v4f v;
#pragma unroll
                for (int m = 0; m < 4; ++m) v[m] = strip[(rl + m) * WT + (cl ^ swz(rl))];
                const size_t moff = (size_t)col * B + row;
                if (Cb) *reinterpret_cast<v4f*>(Cb + moff) = v;
                if (Hb || Lb) {
                    v4s h;
#pragma unroll
                    for (int m = 0; m < 4; ++m) h[m] = H::from_float(v[m]);
                    if (Hb) *reinterpret_cast<v4s*>(Hb + moff) = h;
                    if (Lb) {                     // split modes only: the plain product pays nothing for them
                        v4s lo;
                        float rest[4];
#pragma unroll
                        for (int m = 0; m < 4; ++m) {
                            rest[m] = v[m] - H::to_float(h[m]);
                            lo[m] = H::from_float(rest[m] * lo_scale);
                        }
                        *reinterpret_cast<v4s*>(Lb + moff) = lo;
                        if (L2b) {
                            v4s lo2;
#pragma unroll
                            for (int m = 0; m < 4; ++m) lo2[m] = H::from_float(rest[m] - H::to_float(lo[m]));
                            *reinterpret_cast<v4s*>(L2b + moff) = lo2;
                        }
                    }
                }
                if (H2b) {
                    v4s h2;
#pragma unroll
                    for (int m = 0; m < 4; ++m) h2[m] = H::from_float(a2 * v[m]);
                    *reinterpret_cast<v4s*>(H2b + moff) = h2;
                    if (H2lb) {
                        v4s lo, lo2;
#pragma unroll
                        for (int m = 0; m < 4; ++m) {
                            const float rest = a2 * v[m] - H::to_float(h2[m]);
                            lo[m] = H::from_float(rest * lo_scale);
                            lo2[m] = H::from_float(rest - H::to_float(lo[m]));    // (three planes: lo_scale is 1)
                        }
                        *reinterpret_cast<v4s*>(H2lb + moff) = lo;
                        if (H2l2b) *reinterpret_cast<v4s*>(H2l2b + moff) = lo2;
                    }
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
    });
    if (g.nonfinite && pi == 0 && bad) g.nonfinite[blk] = 1;
}

template <typename H, int TILE>
hipError_t hlaunch_tile(const GemmLaunch& g, hipStream_t stream) {
    const int tiles = g.B / TILE;
    const int64_t W = g.nblocks * g.nprob * (g.sym ? tiles * (tiles + 1) / 2 : tiles * tiles);
    if (W <= 0) return hipSuccess;
    if (W > 0x7fffffffLL) return hipErrorInvalidValue;
    const int ta = g.prob[0].transA, tb = g.prob[0].transB;
    dim3 grid((unsigned)W), block(HCfg<TILE>::NT);
    if (!ta && !tb) hipLaunchKernelGGL((gemm_half_kernel<H, TILE, false, false>), grid, block, 0, stream, g);
    else if (!ta && tb) hipLaunchKernelGGL((gemm_half_kernel<H, TILE, false, true>), grid, block, 0, stream, g);
    else if (ta && !tb) hipLaunchKernelGGL((gemm_half_kernel<H, TILE, true, false>), grid, block, 0, stream, g);
    else hipLaunchKernelGGL((gemm_half_kernel<H, TILE, true, true>), grid, block, 0, stream, g);
    return hipGetLastError();
}

}  // namespace

// tile edge of a 16-bit launch: 256 when the block edge allows it and the launch still gives half the CUs a
// workgroup (a 256 tile on half the chip beats 128 tiles on all of it: 4 x 2048 Clenshaw 3.36 -> 3.00 ms,
// Newton-DB on 16 to 24 blocks of 1024 4 % faster), else as the fp32 kernel.  (A 256 tile of four wavefronts with 128 x 128 each, accumulators in
// AGPRs, was also built: one wavefront per SIMD cannot hide its own latencies, 500-560 TFLOP/s.)
int gemm_half_tile_edge(const GemmLaunch& g) {
    const int64_t t = g.B / 256;
    if (g.B % 256 == 0 && g.nblocks * g.nprob * (g.sym ? t * (t + 1) / 2 : t * t) >= H256_MIN_WORKGROUPS) return 256;
    return gemm_tile_edge(g);
}

static hipError_t launch_half_edge(const GemmLaunch& g, int edge, hipStream_t stream);

// A 256 tile fills a CU, so a launch runs in rounds of 256 workgroups.  A launch of a split mode (several K
// segments per product: long enough to pay for a second launch) whose last round would be at most half full
// (the symmetric residual on 32 blocks: 320 workgroups) computes the blocks of the whole rounds with 256 tiles
// and the remaining blocks with 128 tiles in a second launch.  Returns the number of blocks of the first part
// (nblocks: no split).
int64_t gemm_half_split_blocks(const GemmLaunch& g) {
    if (g.half == HALF_NONE || gemm_half_tile_edge(g) != 256 || !g.prob[0].A2) return g.nblocks;
    const int64_t t = g.B / 256, per_block = g.nprob * (g.sym ? t * (t + 1) / 2 : t * t), W = g.nblocks * per_block;
    const int64_t rem = W % 256;
    const int64_t n_main = (W - rem) / per_block;
    if (W > 256 && rem > 0 && rem <= 128 && n_main >= 1 && n_main < g.nblocks) return n_main;
    return g.nblocks;
}

hipError_t launch_gemm_half(const GemmLaunch& g, hipStream_t stream) {
    const int edge = gemm_half_tile_edge(g);
    const int64_t n_main = gemm_half_split_blocks(g);
    if (n_main < g.nblocks) {
        GemmLaunch a = g, b = g;
        a.nblocks = n_main;
        b.blk0 = g.blk0 + n_main;
        b.nblocks = g.nblocks - n_main;
        hipError_t e = launch_half_edge(a, 256, stream);
        if (e != hipSuccess) return e;
        return launch_half_edge(b, 128, stream);
    }
    return launch_half_edge(g, edge, stream);
}

static hipError_t launch_half_edge(const GemmLaunch& g, int edge, hipStream_t stream) {
    if (g.half == HALF_BF16)
        return edge == 256 ? hlaunch_tile<Bf16, 256>(g, stream)
                           : edge == 128 ? hlaunch_tile<Bf16, 128>(g, stream) : hlaunch_tile<Bf16, 64>(g, stream);
    if (g.half == HALF_FP16)
        return edge == 256 ? hlaunch_tile<Fp16, 256>(g, stream)
                           : edge == 128 ? hlaunch_tile<Fp16, 128>(g, stream) : hlaunch_tile<Fp16, 64>(g, stream);
    return hipErrorInvalidValue;
}

}  // namespace dash
