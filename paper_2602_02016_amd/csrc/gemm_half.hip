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
// for the 256 tile), K slabs of 64 double-buffered in LDS, next slab prefetched into registers,
// LDS-staged epilogue, XCD-aware 1-D grid.  An MFMA operand wants per lane eight consecutive k
// of one row:
//   KC  [row][k]  k contiguous in global memory: rows of 64 elements (pitch 72), one 16-byte
//       LDS read per MFMA operand;
//   K8  [k/8][row][8]  row contiguous in global memory: a thread loads the same eight rows of
//       2, 4 or 8 consecutive k-lines, transposes them in registers and stores, per row, its
//       consecutive k (4, 8 or 16 bytes) into a swizzled 16-byte cell; an MFMA operand is
//       again one 16-byte LDS read.
#include "kernels.h"

#include <utility>

namespace dash {

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

#ifndef DASH_HBK
#define DASH_HBK 64
#endif
constexpr int HBK = DASH_HBK;         // K slab (16-bit elements): 32 or 64
constexpr int HKC_PITCH = HBK + 8;    // elements per row in the KC layout (8 of padding)
constexpr int HKQ = HBK / 8;          // 16-byte vectors per row of a KC slab
// workgroup shape per tile edge: WC x WC wavefronts, each computing a WT x WT part of the tile
//   TILE  64: 2 x 2 wavefronts of 32 x 32   (256 threads)
//   TILE 128: 2 x 2 wavefronts of 64 x 64   (256 threads, two workgroups per CU)
//   TILE 256: 4 x 4 wavefronts of 64 x 64  (1024 threads, one workgroup per CU: the same four wavefronts
//             per SIMD as two 128 tiles, but every operand panel fetched from L2 serves twice the flops)
template <int TILE>
struct HCfg {
    static constexpr int WT = TILE == 64 ? 32 : 64;
    static constexpr int WC = TILE / WT;
    static constexpr int NT = 64 * WC * WC;
    static constexpr int OCC = TILE == 256 ? 1 : 2;        // workgroups per CU the kernel is built for
};
constexpr int HNUM_XCD = 8;

// 16-byte vectors a thread carries per operand slab
template <int TILE>
struct HRegs {
    static constexpr int NV = TILE * HKQ / HCfg<TILE>::NT;
};

template <int TILE>
struct HLds {
    static constexpr int KC_BYTES = TILE * HKC_PITCH * 2;
    static constexpr int K8_BYTES = HKQ * TILE * 16;
    static constexpr int BYTES = KC_BYTES > K8_BYTES ? KC_BYTES : K8_BYTES;
};

// The K8 path (operand stored row-contiguous in global memory, i.e. k is the slow index): a thread owns
// LINES consecutive k-lines x 8 consecutive rows.  TILE/8 row groups x 8/LINES line groups x HBK/8
// k-groups = 256 threads.
template <int TILE>
struct HK8 {
    static constexpr int LINES = HRegs<TILE>::NV;  // 2, 4, 2 for TILE 256, 128, 64
    static constexpr int GPL = TILE / 8;           // 8-row groups per k-line
    static constexpr int SUBS = 8 / LINES;         // line groups per group of 8 k
    static_assert(GPL * SUBS * HKQ == HCfg<TILE>::NT, "K8 decomposition must cover the workgroup");
};

// A slab is TILE*HBK 16-bit elements = TILE*HKQ 16-byte vectors; a thread carries NV of them.  Their byte
// offsets inside the block, without the part that moves with the slab, are fixed for the whole tile: they are
// computed once (32 bits suffice: a block has at most 16384^2 * 2 bytes) and every load is "uniform base of
// the slab + per-thread offset", which keeps the address arithmetic out of the K loop.
template <int TILE, bool KC>
__device__ __forceinline__ void hslab_offsets(int ld, int row0, unsigned (&off)[HRegs<TILE>::NV]) {
    constexpr int NV = HRegs<TILE>::NV;
    const int t = threadIdx.x;
    if (KC) {           // element (row, k) at base[row*ld + k]: HKQ vectors per row
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            const int f = t + HCfg<TILE>::NT * u;
            const int row = f / HKQ, kq = f % HKQ;
            off[u] = ((unsigned)(row0 + row) * (unsigned)ld + 8u * kq) * 2u;
        }
    } else {            // element (row, k) at base[k*ld + row]
        typedef HK8<TILE> U;
        const int rg = t % U::GPL, sub = (t / U::GPL) % U::SUBS, kg = t / (U::GPL * U::SUBS);
#pragma unroll
        for (int l = 0; l < U::LINES; ++l)
            off[l] = ((unsigned)(8 * kg + U::LINES * sub + l) * (unsigned)ld + row0 + 8u * rg) * 2u;
    }
}

// uniform byte offset of slab k0 inside the block
template <bool KC>
__device__ __forceinline__ size_t hslab_base(int ld, int k0) {
    return KC ? (size_t)k0 * 2 : (size_t)k0 * ld * 2;
}

template <int TILE>
__device__ __forceinline__ void hload_slab(const char* __restrict__ slab, const unsigned (&off)[HRegs<TILE>::NV],
                                           v4u (&r)[HRegs<TILE>::NV]) {
#pragma unroll
    for (int u = 0; u < HRegs<TILE>::NV; ++u) r[u] = *reinterpret_cast<const v4u*>(slab + off[u]);
}

// K8 layout in LDS: [k/8][row'][8 k], 16 bytes per (k-group, row), row' = row ^ ((row / 8) % 8): the
// swizzle spreads the eight rows one thread writes at stride 128 bytes over all banks, and keeps 32
// consecutive rows inside the same 512 bytes, so an MFMA operand (eight consecutive k of one row) is
// one conflict-free 16-byte read per lane, exactly as in the KC layout.
template <int TILE, bool KC>
__device__ __forceinline__ void hstore_slab(char* __restrict__ s, const v4u (&r)[HRegs<TILE>::NV]) {
    constexpr int NV = HRegs<TILE>::NV;
    const int t = threadIdx.x;
    if (KC) {
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            const int f = t + HCfg<TILE>::NT * u;
            const int row = f / HKQ, kq = f % HKQ;
            *reinterpret_cast<v4u*>(s + (row * HKC_PITCH + 8 * kq) * 2) = r[u];
        }
    } else {
        typedef HK8<TILE> U;
        const int rg = t % U::GPL, sub = (t / U::GPL) % U::SUBS, kg = t / (U::GPL * U::SUBS);
        char* d = s + (kg * TILE + 8 * rg) * 16 + sub * U::LINES * 2;
#pragma unroll
        for (int i = 0; i < 8; ++i) {       // row 8*rg + i: its LINES consecutive k, two per dword
            unsigned int w[U::LINES / 2];
#pragma unroll
            for (int kp = 0; kp < U::LINES / 2; ++kp) {
                const unsigned int a = r[2 * kp][i / 2], b = r[2 * kp + 1][i / 2];
                w[kp] = (i & 1) ? ((a >> 16) | (b & 0xffff0000u)) : ((a & 0xffffu) | (b << 16));
            }
            char* q = d + ((i ^ (rg & 7)) * 16);
            if (U::LINES == 8) {
                v4u v; v[0] = w[0]; v[1] = w[1 % (U::LINES / 2)]; v[2] = w[2 % (U::LINES / 2)]; v[3] = w[3 % (U::LINES / 2)];
                *reinterpret_cast<v4u*>(q) = v;
            } else if (U::LINES == 4) {
                typedef unsigned int v2u __attribute__((ext_vector_type(2)));
                v2u v; v[0] = w[0]; v[1] = w[1 % (U::LINES / 2)];
                *reinterpret_cast<v2u*>(q) = v;
            } else {
                *reinterpret_cast<unsigned int*>(q) = w[0];
            }
        }
    }
}

// operand of MFMA step `st` (16 k each) for the 32-row sub-tile at r0:
// element (r0 + lane%32, 16*st + 8*(lane/32) + 0..7)
template <int TILE, bool KC>
__device__ __forceinline__ v4u hread_frag(const char* __restrict__ s, int r0, int st, int lane) {
    const int rr = r0 + (lane & 31);
    if (KC) return *reinterpret_cast<const v4u*>(s + (rr * HKC_PITCH + 16 * st + 8 * (lane >> 5)) * 2);
    return *reinterpret_cast<const v4u*>(s + ((2 * st + (lane >> 5)) * TILE + (rr ^ ((rr >> 3) & 7))) * 16);
}

template <typename H, int TILE, bool TA, bool TB>
__global__ __launch_bounds__(HCfg<TILE>::NT, HCfg<TILE>::OCC) void gemm_half_kernel(GemmLaunch g) {
    constexpr int MT = HCfg<TILE>::WT / 32;
    constexpr bool A_KC = !TA;
    constexpr bool B_KC = TB;
    constexpr int NV = HRegs<TILE>::NV;
    constexpr int SLAB = HLds<TILE>::BYTES;

    __shared__ __attribute__((aligned(16))) char lds[2 * 2 * SLAB];

    const int64_t W = gridDim.x;
    const int64_t bid = blockIdx.x;
    const int64_t xcd = bid % HNUM_XCD, local = bid / HNUM_XCD;
    const int64_t per = W / HNUM_XCD, rem = W % HNUM_XCD;
    const int64_t lid = xcd * per + (xcd < rem ? xcd : rem) + local;

    const int B = g.B;
    const int tiles = B / TILE;
    const int T = g.sym ? tiles * (tiles + 1) / 2 : tiles * tiles;
    const int64_t blk = lid / ((int64_t)g.nprob * T);
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
    const int nseg = P.A2 ? 3 : 1;
    const u16* __restrict__ Ahi = static_cast<const u16*>(P.A) + boff;
    const u16* __restrict__ Bhi = static_cast<const u16*>(P.B) + boff;
    const u16* __restrict__ Alo = P.A2 ? static_cast<const u16*>(P.A2) + boff : Ahi;
    const u16* __restrict__ Blo = P.B2 ? static_cast<const u16*>(P.B2) + boff : Bhi;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
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
    v4u ra[NV], rb[NV];
    unsigned offa[NV], offb[NV];
    hslab_offsets<TILE, A_KC>(B, row0, offa);
    hslab_offsets<TILE, B_KC>(B, col0, offb);
    // The slabs are requested in order, segment after segment (the small terms are summed first:
    // A_lo B_hi, A_hi B_lo, A_hi B_hi; a plain product is the last segment alone).  The uniform base
    // addresses of the next slab are carried along and stepped, so the K loop holds no address set-up.
    const size_t stepa = hslab_base<A_KC>(B, HBK), stepb = hslab_base<B_KC>(B, HBK);
    int seg_next = nseg == 1 ? 2 : 0, ks_next = 0;
    const char* pa = reinterpret_cast<const char*>(seg_next == 0 ? Alo : Ahi);
    const char* pb = reinterpret_cast<const char*>(Bhi);
    auto load_next = [&]() {
        hload_slab<TILE>(pa, offa, ra);
        hload_slab<TILE>(pb, offb, rb);
        if (++ks_next < KS) {
            pa += stepa;
            pb += stepb;
        } else {
            ks_next = 0;
            ++seg_next;
            pa = reinterpret_cast<const char*>(Ahi);
            pb = reinterpret_cast<const char*>(seg_next == 1 ? Blo : Bhi);
        }
    };
    // multiply slab kt out of its LDS buffer
    auto compute = [&](auto BUF) {
        const char* sa = lds + decltype(BUF)::value * 2 * SLAB;
        const char* sb = sa + SLAB;
        // operand fragments of step st+1 are requested from LDS before the MFMAs of step st issue
        v4u fa[2][MT], fb[2][MT];
#pragma unroll
        for (int i = 0; i < MT; ++i) fa[0][i] = hread_frag<TILE, A_KC>(sa, wm + 32 * i, 0, lane);
#pragma unroll
        for (int j = 0; j < MT; ++j) fb[0][j] = hread_frag<TILE, B_KC>(sb, wn + 32 * j, 0, lane);
#pragma unroll
        for (int st = 0; st < HBK / 16; ++st) {
            const int cur = st & 1, nxt = cur ^ 1;
            if (st + 1 < HBK / 16) {
#pragma unroll
                for (int i = 0; i < MT; ++i) fa[nxt][i] = hread_frag<TILE, A_KC>(sa, wm + 32 * i, st + 1, lane);
#pragma unroll
                for (int j = 0; j < MT; ++j) fb[nxt][j] = hread_frag<TILE, B_KC>(sb, wn + 32 * j, st + 1, lane);
            }
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int j = 0; j < MT; ++j)
                    acc[i][j] = H::mfma(fa[cur][i], fb[cur][j], acc[i][j]);
        }
    };
    load_next();
    hstore_slab<TILE, A_KC>(lds, ra);
    hstore_slab<TILE, B_KC>(lds + SLAB, rb);
    __syncthreads();
    // one iteration per slab; the loop is unrolled by two so that the LDS buffer of a slab is a compile-time
    // constant and every LDS address is "per-thread base + immediate"
    auto iteration = [&](int kt, auto BUF) {
        const bool more = kt + 1 < KT;
        if (more) load_next();           // next slab into registers while this one is multiplied
        compute(BUF);
        if (more) {
            char* da = lds + (1 - decltype(BUF)::value) * 2 * SLAB;
            hstore_slab<TILE, A_KC>(da, ra);
            hstore_slab<TILE, B_KC>(da + SLAB, rb);
        }
        __syncthreads();
    };
    for (int kt = 0; kt < KT; kt += 2) {
        iteration(kt, std::integral_constant<int, 0>{});
        if (kt + 1 < KT) iteration(kt + 1, std::integral_constant<int, 1>{});
    }

    // ---- epilogue, staged through LDS (free after the last barrier of the main loop) ----
    // The MFMA leaves a lane with one column and scattered rows; storing from there means 4-byte (or
    // 2-byte) stores and a fully unrolled epilogue whose code no longer fits the instruction cache.
    // Instead every wavefront passes its accumulators, one strip of 32 rows x WT columns at a time,
    // through a private LDS region and comes back with row-contiguous quads: 16-byte loads of D,
    // 16-byte stores of fp32 outputs, 8-byte stores of 16-bit outputs, in a compact loop.
    const float mult = P.mult ? P.mult[blk] : 1.f;
    const float alpha = P.alpha * mult, beta = P.beta * mult, gamma = P.gamma * mult;
    const float* __restrict__ Db = P.D ? P.D + boff : nullptr;
    float* __restrict__ Cb = P.C ? P.C + boff : nullptr;
    u16* __restrict__ Hb = P.Ch ? static_cast<u16*>(P.Ch) + boff : nullptr;
    u16* __restrict__ H2b = P.C2h ? static_cast<u16*>(P.C2h) + boff : nullptr;
    u16* __restrict__ Lb = P.Cl ? static_cast<u16*>(P.Cl) + boff : nullptr;    // low plane of the result
    const float a2 = P.a2, g2 = P.g2;
    // symmetric mode: an off-diagonal tile is also written transposed
    const bool mirror = g.sym && ti != tj;
    constexpr int WT = HCfg<TILE>::WT;            // columns of a wavefront's strip
    constexpr int SP = WT + 4;                    // strip pitch in floats
    constexpr int QPR = WT / 4;                   // quads per strip row
    constexpr int RPI = 64 / QPR;                 // strip rows one pass of the wavefront covers
    static_assert((HCfg<TILE>::NT / 64) * 32 * SP * 4 <= 4 * SLAB, "strips must fit the operand buffers");
    float* strip = reinterpret_cast<float*>(lds) + wave * 32 * SP;
    bool bad = false;
    static_for<MT>([&](auto I) {
        constexpr int i = decltype(I)::value;
        // phase A: alpha * acc into the strip, element (8q + 4(lane/32) + m, 32j + lane%32)
        static_for<MT>([&](auto J) {
            constexpr int j = decltype(J)::value;
#pragma unroll
            for (int r = 0; r < 16; ++r)
                strip[(8 * (r / 4) + 4 * (lane >> 5) + (r % 4)) * SP + 32 * j + (lane & 31)] = alpha * acc[i][j][r];
        });
        __syncthreads();
        // phase B: row-contiguous quads
        const int rbase = row0 + wm + 32 * i, cbase = col0 + wn;
#pragma unroll 1
        for (int t = 0; t < 32 / RPI; ++t) {
            const int rl = lane / QPR + RPI * t, c = (lane % QPR) * 4;
            v4f v = *reinterpret_cast<const v4f*>(strip + rl * SP + c);
            const int row = rbase + rl, col = cbase + c;
            const size_t off = (size_t)row * B + col;
            if (Db) {
                const v4f d = *reinterpret_cast<const v4f*>(Db + off);
#pragma unroll
                for (int m = 0; m < 4; ++m) v[m] += beta * d[m];
            }
            v4s h, h2, lo;
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                if (row == col + m) v[m] += gamma;
                bad |= !(fabsf(v[m]) <= 3.0e38f);
                h[m] = H::from_float(v[m]);
                lo[m] = H::from_float(v[m] - H::to_float(h[m]));
                h2[m] = H::from_float(a2 * v[m] + (row == col + m ? g2 : 0.f));
            }
            if (Cb) *reinterpret_cast<v4f*>(Cb + off) = v;
            if (Hb) *reinterpret_cast<v4s*>(Hb + off) = h;
            if (Lb) *reinterpret_cast<v4s*>(Lb + off) = lo;
            if (H2b) *reinterpret_cast<v4s*>(H2b + off) = h2;
            if (mirror) *reinterpret_cast<v4f*>(strip + rl * SP + c) = v;     // final values for phase C
        }
        __syncthreads();
        // phase C (mirrored tiles only): back in the MFMA layout a lane holds four consecutive rows of
        // one column = four consecutive elements of a row of the transposed tile
        if (mirror) {
#pragma unroll 1
            for (int jq = 0; jq < MT * 4; ++jq) {
                const int j = jq >> 2, q = jq & 3;
                const int rl = 8 * q + 4 * (lane >> 5), cl = 32 * j + (lane & 31);
                const int row = rbase + rl, col = cbase + cl;
                v4f v;
                v4s h, h2, lo;
#pragma unroll
                for (int m = 0; m < 4; ++m) {
                    v[m] = strip[(rl + m) * SP + cl];
                    h[m] = H::from_float(v[m]);
                    lo[m] = H::from_float(v[m] - H::to_float(h[m]));
                    h2[m] = H::from_float(a2 * v[m] + (row + m == col ? g2 : 0.f));
                }
                const size_t moff = (size_t)col * B + row;
                if (Cb) *reinterpret_cast<v4f*>(Cb + moff) = v;
                if (Hb) *reinterpret_cast<v4s*>(Hb + moff) = h;
                if (Lb) *reinterpret_cast<v4s*>(Lb + moff) = lo;
                if (H2b) *reinterpret_cast<v4s*>(H2b + moff) = h2;
            }
            __syncthreads();
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

// tile edge of a 16-bit launch: 256 when the block edge allows it and the launch still gives every CU a
// workgroup, else as the fp32 kernel.  (A 256 tile of four wavefronts with 128 x 128 each, accumulators in
// AGPRs, was also built: one wavefront per SIMD cannot hide its own latencies, 500-560 TFLOP/s.)
int gemm_half_tile_edge(const GemmLaunch& g) {
#ifndef DASH_NO_TILE256
    const int64_t t = g.B / 256;
    if (g.B % 256 == 0 && g.nblocks * g.nprob * (g.sym ? t * (t + 1) / 2 : t * t) >= 256) return 256;
#endif
    return gemm_tile_edge(g);
}

hipError_t launch_gemm_half(const GemmLaunch& g, hipStream_t stream) {
    const int edge = gemm_half_tile_edge(g);
    if (g.half == HALF_BF16)
        return edge == 256 ? hlaunch_tile<Bf16, 256>(g, stream)
                           : edge == 128 ? hlaunch_tile<Bf16, 128>(g, stream) : hlaunch_tile<Bf16, 64>(g, stream);
    if (g.half == HALF_FP16)
        return edge == 256 ? hlaunch_tile<Fp16, 256>(g, stream)
                           : edge == 128 ? hlaunch_tile<Fp16, 128>(g, stream) : hlaunch_tile<Fp16, 64>(g, stream);
    return hipErrorInvalidValue;
}

}  // namespace dash
