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
// Same decomposition as the fp32 kernel: 256 threads, 2 x 2 wavefronts, TILE x TILE per
// workgroup, K slabs of 32 double-buffered in LDS, next slab prefetched into registers,
// XCD-aware 1-D grid.  An MFMA operand wants per lane eight consecutive k of one row:
//   KC  [row][k]  k contiguous in global memory: rows of 32 bf16 (pitch 40), one 16-byte
//       LDS read per MFMA operand;
//   RC2 [k/2][row][2]  row contiguous in global memory: a thread loads the same eight
//       columns of two consecutive k-lines, interleaves them into dwords {k even, k odd}
//       and stores 32 contiguous bytes; an MFMA operand is four 4-byte reads at
//       consecutive addresses across lanes (pitch TILE+8 dwords).
#include "kernels.h"

namespace dash {

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
constexpr int HNT = 256;
constexpr int HNUM_XCD = 8;

// 16-byte vectors a thread carries per operand slab (the RC2 path needs two per unit)
template <int TILE>
struct HRegs {
    static constexpr int NV = TILE * HKQ / HNT < 2 ? 2 : TILE * HKQ / HNT;
};

template <int TILE>
struct HLds {
    static constexpr int RC_PITCH = TILE + 8;                 // dwords per k-pair line
    static constexpr int KC_BYTES = TILE * HKC_PITCH * 2;
    static constexpr int RC_BYTES = (HBK / 2) * RC_PITCH * 4;
    static constexpr int BYTES = KC_BYTES > RC_BYTES ? KC_BYTES : RC_BYTES;
};

// A slab is TILE*32 bf16 = TILE*4 16-byte vectors; a thread carries TILE*4/256 of them.
template <int TILE, bool KC>
__device__ __forceinline__ void hload_slab(const u16* __restrict__ base, int ld, int row0, int k0,
                                           v4u (&r)[HRegs<TILE>::NV]) {
    constexpr int NV = TILE * HKQ / HNT;
    const int t = threadIdx.x;
    if (KC) {           // element (row, k) at base[row*ld + k]: 4 vectors per row
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            const int f = t + HNT * u;
            const int row = f / HKQ, kq = f % HKQ;
            r[u] = *reinterpret_cast<const v4u*>(base + (size_t)(row0 + row) * ld + k0 + 8 * kq);
        }
    } else {            // element (row, k) at base[k*ld + row]: unit = 2 k-lines x 8 rows
        constexpr int GPL = TILE / 8;       // 8-row groups per k-line
        constexpr int UNITS = (HBK / 2) * GPL;
#pragma unroll
        for (int u = 0; u < (UNITS + HNT - 1) / HNT; ++u) {
            const int f = t + HNT * u;
            if (f < UNITS) {
                const int q = f / GPL, rg = f % GPL;
                const u16* p = base + (size_t)(k0 + 2 * q) * ld + row0 + 8 * rg;
                r[2 * u] = *reinterpret_cast<const v4u*>(p);
                r[2 * u + 1] = *reinterpret_cast<const v4u*>(p + ld);
            }
        }
    }
}

template <int TILE, bool KC>
__device__ __forceinline__ void hstore_slab(char* __restrict__ s, const v4u (&r)[HRegs<TILE>::NV]) {
    constexpr int NV = TILE * HKQ / HNT;
    const int t = threadIdx.x;
    if (KC) {
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            const int f = t + HNT * u;
            const int row = f / HKQ, kq = f % HKQ;
            *reinterpret_cast<v4u*>(s + (row * HKC_PITCH + 8 * kq) * 2) = r[u];
        }
    } else {
        constexpr int GPL = TILE / 8;
        constexpr int UNITS = (HBK / 2) * GPL;
        constexpr int P = HLds<TILE>::RC_PITCH;
#pragma unroll
        for (int u = 0; u < (UNITS + HNT - 1) / HNT; ++u) {
            const int f = t + HNT * u;
            if (f >= UNITS) continue;
            const int q = f / GPL, rg = f % GPL;
            const v4u a = r[2 * u], b = r[2 * u + 1];   // k even line, k odd line; each dword = rows (2i, 2i+1)
            v4u lo, hi;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                lo[2 * i] = (a[i] & 0xffffu) | (b[i] << 16);
                lo[2 * i + 1] = (a[i] >> 16) | (b[i] & 0xffff0000u);
                hi[2 * i] = (a[i + 2] & 0xffffu) | (b[i + 2] << 16);
                hi[2 * i + 1] = (a[i + 2] >> 16) | (b[i + 2] & 0xffff0000u);
            }
            unsigned int* d = reinterpret_cast<unsigned int*>(s) + q * P + 8 * rg;
            *reinterpret_cast<v4u*>(d) = lo;
            *reinterpret_cast<v4u*>(d + 4) = hi;
        }
    }
}

// operand of MFMA step `st` (16 k each) for the 32-row sub-tile at r0:
// element (r0 + lane%32, 16*st + 8*(lane/32) + 0..7)
template <int TILE, bool KC>
__device__ __forceinline__ v4u hread_frag(const char* __restrict__ s, int r0, int st, int lane) {
    const int rr = r0 + (lane & 31), kh = 16 * st + 8 * (lane >> 5);
    v4u x;
    if (KC) {
        x = *reinterpret_cast<const v4u*>(s + (rr * HKC_PITCH + kh) * 2);
    } else {
        constexpr int P = HLds<TILE>::RC_PITCH;
        const unsigned int* d = reinterpret_cast<const unsigned int*>(s) + (kh >> 1) * P + rr;
        x[0] = d[0];
        x[1] = d[P];
        x[2] = d[2 * P];
        x[3] = d[3 * P];
    }
    return x;
}

template <typename H, int TILE, bool TA, bool TB>
__global__ __launch_bounds__(HNT, 2) void gemm_half_kernel(GemmLaunch g) {
    constexpr int MT = TILE / 64;
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
    const int wm = (wave >> 1) * (TILE / 2), wn = (wave & 1) * (TILE / 2);

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
    // slab kk belongs to segment kk / KS; the small terms are summed first
    auto load = [&](int kk) {
        const int seg = nseg == 1 ? 2 : kk / KS, k0 = (kk % KS) * HBK;
        const u16* __restrict__ Ab = seg == 0 ? Alo : Ahi;
        const u16* __restrict__ Bb = seg == 1 ? Blo : Bhi;
        hload_slab<TILE, A_KC>(Ab, B, row0, k0, ra);
        hload_slab<TILE, B_KC>(Bb, B, col0, k0, rb);
    };
    load(0);
    hstore_slab<TILE, A_KC>(lds, ra);
    hstore_slab<TILE, B_KC>(lds + SLAB, rb);
    __syncthreads();

    for (int kt = 0; kt < KT; ++kt) {
        const char* sa = lds + (kt & 1) * 2 * SLAB;
        const char* sb = sa + SLAB;
        const bool more = kt + 1 < KT;
        if (more) load(kt + 1);
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
        if (more) {
            char* da = lds + ((kt + 1) & 1) * 2 * SLAB;
            hstore_slab<TILE, A_KC>(da, ra);
            hstore_slab<TILE, B_KC>(da + SLAB, rb);
        }
        __syncthreads();
    }

    const float mult = P.mult ? P.mult[blk] : 1.f;
    const float alpha = P.alpha * mult, beta = P.beta * mult, gamma = P.gamma * mult;
    const float* __restrict__ Db = P.D ? P.D + boff : nullptr;
    float* __restrict__ Cb = P.C ? P.C + boff : nullptr;
    u16* __restrict__ Hb = P.Ch ? static_cast<u16*>(P.Ch) + boff : nullptr;
    u16* __restrict__ H2b = P.C2h ? static_cast<u16*>(P.C2h) + boff : nullptr;
    u16* __restrict__ Lb = P.Cl ? static_cast<u16*>(P.Cl) + boff : nullptr;    // low plane of the result
    const float a2 = P.a2, g2 = P.g2;
    // symmetric mode: an off-diagonal tile is also written transposed (four consecutive rows
    // of one column = four consecutive elements of a row of the transposed tile)
    const bool mirror = g.sym && ti != tj;
    bool bad = false;
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < MT; ++j) {
            const int col = col0 + wn + 32 * j + (lane & 31);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int rbase = row0 + wm + 32 * i + 8 * q + 4 * (lane >> 5);
                v4f out;
                v4s outh, outh2, outl;
#pragma unroll
                for (int m = 0; m < 4; ++m) {
                    const int row = rbase + m;
                    const size_t off = (size_t)row * B + col;
                    float v = alpha * acc[i][j][4 * q + m];
                    if (Db) v += beta * Db[off];
                    if (row == col) v += gamma;
                    bad |= !(fabsf(v) <= 3.0e38f);
                    out[m] = v;
                    outh[m] = H::from_float(v);
                    if (Cb) Cb[off] = v;
                    if (Hb) Hb[off] = outh[m];
                    if (Lb) {
                        outl[m] = H::from_float(v - H::to_float(outh[m]));
                        Lb[off] = outl[m];
                    }
                    if (H2b) {
                        outh2[m] = H::from_float(a2 * v + (row == col ? g2 : 0.f));
                        H2b[off] = outh2[m];
                    }
                }
                if (mirror) {
                    const size_t moff = (size_t)col * B + rbase;
                    if (Cb) *reinterpret_cast<v4f*>(Cb + moff) = out;
                    if (Hb) *reinterpret_cast<v4s*>(Hb + moff) = outh;
                    if (Lb) *reinterpret_cast<v4s*>(Lb + moff) = outl;
                    if (H2b) *reinterpret_cast<v4s*>(H2b + moff) = outh2;
                }
            }
        }
    if (g.nonfinite && pi == 0 && bad) g.nonfinite[blk] = 1;
}

template <typename H, int TILE>
hipError_t hlaunch_tile(const GemmLaunch& g, hipStream_t stream) {
    const int tiles = g.B / TILE;
    const int64_t W = g.nblocks * g.nprob * (g.sym ? tiles * (tiles + 1) / 2 : tiles * tiles);
    if (W <= 0) return hipSuccess;
    if (W > 0x7fffffffLL) return hipErrorInvalidValue;
    const int ta = g.prob[0].transA, tb = g.prob[0].transB;
    dim3 grid((unsigned)W), block(HNT);
    if (!ta && !tb) hipLaunchKernelGGL((gemm_half_kernel<H, TILE, false, false>), grid, block, 0, stream, g);
    else if (!ta && tb) hipLaunchKernelGGL((gemm_half_kernel<H, TILE, false, true>), grid, block, 0, stream, g);
    else if (ta && !tb) hipLaunchKernelGGL((gemm_half_kernel<H, TILE, true, false>), grid, block, 0, stream, g);
    else hipLaunchKernelGGL((gemm_half_kernel<H, TILE, true, true>), grid, block, 0, stream, g);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_half(const GemmLaunch& g, hipStream_t stream) {
    const bool big = gemm_tile_edge(g) == 128;
    if (g.half == HALF_BF16) return big ? hlaunch_tile<Bf16, 128>(g, stream) : hlaunch_tile<Bf16, 64>(g, stream);
    if (g.half == HALF_FP16) return big ? hlaunch_tile<Fp16, 128>(g, stream) : hlaunch_tile<Fp16, 64>(g, stream);
    return hipErrorInvalidValue;
}

}  // namespace dash
