// Internal launch interface between the host-side library (dash.hip) and the kernels.
// Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dash {

// One batched product  C_b = mult_b * (alpha * op(A_b) op(B_b) + beta * D_b + gamma * I).
// mult (per-block factor, device array) may be null (= 1).  D may be null when beta == 0
// and may equal C.
// fp32 launches: A, B are fp32 stacks, Ch and C2h are ignored.
// 16-bit launches (GemmLaunch::half = HALF_BF16 or HALF_FP16): A, B point to bf16 / fp16 stacks
// (same [N][B][B] layout, 2-byte elements); the result is written to C in fp32 (if C is not
// null) and, rounded to the 16-bit format, to Ch (if Ch is not null); D stays fp32; C2 is
// ignored and the second output goes, rounded, to C2h.
enum { HALF_NONE = 0, HALF_BF16 = 1, HALF_FP16 = 2 };

struct GemmProblem {
    const void* A;
    const void* B;
    const float* D;
    float* C;
    void* Ch;
    float* C2;             // fp32 launches: optional second output a2 * C + g2 * I
    void* C2h;             // 16-bit launches: the same second output, rounded to the 16-bit format
    // 16-bit launches, split-operand mode: A, B are the high planes, A2, B2 the low planes (null =
    // plain 16-bit product); Cl receives the low plane of the result (Ch the high plane)
    const void* A2;
    const void* B2;
    void* Cl;
    // three-plane mode: A3, B3 are third (lowest) planes (null = two planes), Cl2 receives the third plane of
    // the result; the product then has six segments (see gemm_half.hip)
    const void* A3;
    const void* B3;
    void* Cl2;
    void* C2l;             // middle and lowest plane of the second output (three-plane mode, with C2h)
    void* C2l2;
    float a2, g2;
    const float* mult;
    float alpha, beta, gamma;
    int transA, transB;
};

// Up to two products over the same block range in one launch (Newton-DB computes
// Y E and E Z together; accumulate computes G G^T and G^T G together).
struct GemmLaunch {
    GemmProblem prob[2];
    int nprob;
    int B;                 // block edge
    int M, N, K;           // 0 = B.  Non-zero: op(A) is M x K, op(B) is K x N, C is M x N per block
                           // (contiguous stacks; fp32 launches only; symmetric mode needs M == N)
    int64_t nblocks;       // blocks in this launch
    int64_t blk0;          // index of the launch's first block inside the stacks the pointers name (normally 0)
    int64_t n_main, w_main;   // filled in by launch_gemm: blocks and workgroups computed with the launch's own tile edge;
                              // the remaining blocks of an fp32 launch are computed with 64 tiles by its last workgroups
    int32_t* nonfinite;    // per-block flag for prob[0]'s output, or null
    int half;              // HALF_NONE: fp32 MFMA operands; HALF_BF16 / HALF_FP16: 16-bit operands
    int sym;               // 1: every product of the launch is symmetric in exact arithmetic:
                           //    only tiles on or above the diagonal are computed, the rest mirrored
};

hipError_t launch_gemm(const GemmLaunch& g, hipStream_t stream);
int gemm_tile_edge(const GemmLaunch& g);          // tile edge launch_gemm picks for fp32 (64 or 128; see gemm_split_blocks)
int gemm_half_tile_edge(const GemmLaunch& g);     // tile edge of a 16-bit launch (64, 128 or 256)
double gemm_tile_fraction(const GemmLaunch& g);   // share of output tiles actually computed
int64_t gemm_split_blocks(const GemmLaunch& g);   // fp32: blocks a launch computes with 128 tiles; the rest (if any) with 64
int64_t gemm_half_split_blocks(const GemmLaunch& g);   // 16-bit: blocks computed with 256 tiles when a launch is split; the rest with 128
hipError_t launch_gemm_half(const GemmLaunch& g, hipStream_t stream);   // gemm_half.hip

// partial[b*P + q] = sum over the q-th row slab of block b of (A + eps I)^2 (mode 0)
// or of the diagonal of (A + eps I) (mode 1).  P = norm_slabs(B).
int norm_slabs(int B);
hipError_t launch_norm_partials(const float* A, int64_t nblocks, int B, float eps, int mode,
                                float* partial, hipStream_t stream);
// s = sqrt(sum partial) (mode 0) | sum partial (mode 1) | 1 (mode 2);
// writes s[b], inv_s[b] = 1/s, unscale[b] = s^(-1/p) (any of the three may be null).
hipError_t launch_finalize_scale(const float* partial, int64_t nblocks, int P, int mode, int p,
                                 float* s, float* inv_s, float* unscale, hipStream_t stream);

// t = (in + eps I) * mult_b ; o1 = a1 * t + g1 * I ; o2 = a2 * o1 + g2 * I.
// o1 is written to out1 (fp32) and/or h1 (rounded to the 16-bit format `half`), o2 to out2 and/or
// h2; any of the four destinations and mult may be null.
hipError_t launch_scale_shift(const float* in, int64_t nblocks, int B, float eps, const float* mult,
                              float a1, float g1, float* out1, float a2, float g2, float* out2,
                              void* h1, void* h2, int32_t* nonfinite, hipStream_t stream, int half = HALF_BF16,
                              void* l1 = nullptr, void* l2 = nullptr,    // l1, l2: low planes of o1, o2 (split mode)
                              void* ll1 = nullptr, void* ll2 = nullptr); // third planes (three-plane mode)

// Multi-Power-Iteration scaling (power_iteration.hip): s_b = 2 * lambda_PI(A_b + eps I) from
// `sweeps` passes over the block with a pool of `pool` (<= 32) start vectors V0 ([B][pool]
// row-major, shared by all blocks).  V, W: scratch of n * B * 32 floats each (kept pool-major, [n][32][B]); q: scratch of
// n * power_iteration_q_floats(B) floats.
size_t power_iteration_bytes_per_block(int B);
size_t power_iteration_q_floats(int B);
hipError_t launch_power_iteration(const float* A, int64_t nblocks, int B, float eps, const float* V0, int pool,
                                  int sweeps, int p, float* V, float* W, float* q, float* s, float* inv_s,
                                  float* unscale, hipStream_t stream);

// 1-D parameters: L_b <- beta L_b + alpha g_b g_b^T (g: [n][B]);  u_b = X_b g_b
hipError_t launch_outer_accumulate(const float* g, float* L, int64_t nblocks, int B, float beta, float alpha,
                                   hipStream_t stream);
hipError_t launch_matvec(const float* X, const float* g, float* u, int64_t nblocks, int B, hipStream_t stream);

// block() of a row-major layer W (leading dimension ld): the nm x nn grid of bm x bn sub-matrices with
// origin (r0, c0) and pitch B in both directions <-> stack [nm*nn][bm][bn] (row-major block order).
// scatter = false: W -> stack; true: stack -> W.
hipError_t launch_block_copy(float* W, float* stack, int64_t ld, int64_t r0, int64_t c0, int B, int bm, int bn,
                             int pm, int pn, int64_t nm, int64_t nn, bool scatter, hipStream_t stream);

hipError_t launch_fill_i32(int32_t* p, int64_t n, int32_t v, hipStream_t stream);

// grafting on blocks of `elems` contiguous floats (elems a multiple of 4 x graft_slabs(elems)):
// Acc <- beta_g Acc + (1-beta_g) G.G ; partial sums of P^2 and U^2 per slab
int graft_slabs(int64_t elems);
hipError_t launch_graft_partials(const float* G, const float* U, float* Acc, int64_t nblocks, int64_t elems,
                                 float beta_g, float eps_g, float* partial /* [n][slabs][2] */,
                                 hipStream_t stream);
// s_b = sqrt(sum P^2 / sum U^2); theta -= lr * s_b * U (theta may be null); scaled = s_b * U (may be null,
// may equal U); s_out may be null
hipError_t launch_graft_apply(const float* U, float* theta, const float* partial, int64_t nblocks,
                              int64_t elems, float lr, float* s_out, float* scaled, hipStream_t stream);
// y -= a * x over n floats (any n; pointers 16-byte aligned)
hipError_t launch_axpy(float* y, const float* x, int64_t n, float a, hipStream_t stream);

}  // namespace dash
