// Multi-Power-Iteration estimate of lambda_max for every block of a stack
// (paper Sections 3.4 and 3.5): a pool of up to 32 start vectors is multiplied by the
// block `sweeps` times, the largest Rayleigh quotient of the last sweep is lambda_PI, and
// the block is scaled by s = 2 * lambda_PI.
//
// One sweep reads the block once (4 B^2 bytes) and is HBM-bound, as the paper notes: the
// pool only widens the skinny product W = A V.  The pool vectors are kept pool-major
// ([32][B] per block: a column of V is contiguous) so that every operand of the sweep is
// read 16 bytes per lane.  Kernels:
//   pi_init    V_b = start vectors with unit columns (pool padded with zero columns to 32)
//   pi_sweep   W_b = A_b V_b + eps V_b with v_mfma_f32_32x32x2_f32.  A workgroup owns 64 rows
//              of A; its four wavefronts split K (32-wide chunks, round robin), each streams its
//              part of the 64 rows straight from global memory into the MFMA A operand (every
//              element of A is used once, so LDS staging would buy nothing) and reuses each
//              chunk of V for both 32-row tiles; the four partial results meet in LDS.  The loads
//              of a wavefront's next chunk are in flight while the MFMAs of the current one run.
//   pi_reduce  per block: q_j = v_j . w_j, V <- W with unit columns; after the last sweep
//              s = 2 max_j q_j, 1/s and s^(-1/p)
// Reductions are per block in a fixed order (no atomics): results do not depend on scheduling.
#include "kernels.h"

namespace dash {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));

namespace {

constexpr int POOL = 32;     // columns of V (pool members beyond the requested count are zero)
constexpr int PNT = 256;

// sum over the 8 consecutive lanes that share a pool column
__device__ __forceinline__ float sum8(float x) {
    x += __shfl_xor(x, 1);
    x += __shfl_xor(x, 2);
    x += __shfl_xor(x, 4);
    return x;
}

// grid = nblocks; V0: [B][m] row-major (shared by all blocks); V: [nblocks][32][B]
__global__ __launch_bounds__(PNT) void pi_init_kernel(const float* __restrict__ V0, int m, int B,
                                                     float* __restrict__ V) {
    __shared__ float part[PNT / POOL][POOL];
    __shared__ float inv_norm[POOL];
    const int j = threadIdx.x % POOL, rg = threadIdx.x / POOL;
    float acc = 0.f;
    if (j < m)
        for (int i = rg; i < B; i += PNT / POOL) { const float x = V0[(size_t)i * m + j]; acc += x * x; }
    part[rg][j] = acc;
    __syncthreads();
    if (rg == 0) {
        float t = 0.f;
        for (int r = 0; r < PNT / POOL; ++r) t += part[r][j];
        inv_norm[j] = t > 0.f ? 1.f / sqrtf(t) : 0.f;
    }
    __syncthreads();
    float* __restrict__ Vb = V + (size_t)blockIdx.x * B * POOL;
    for (int idx = threadIdx.x; idx < POOL * B; idx += PNT) {
        const int c = idx / B, i = idx % B;
        Vb[idx] = c < m ? V0[(size_t)i * m + c] * inv_norm[c] : 0.f;
    }
}

// grid = (B/64, nblocks); the four wavefronts of a workgroup split K
__global__ __launch_bounds__(PNT) void pi_sweep_kernel(const float* __restrict__ A, const float* __restrict__ V,
                                                      float* __restrict__ W, int B, float eps) {
    __shared__ float part[4][2][16][64];          // [wavefront][row tile][accumulator register][lane]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row0 = blockIdx.x * 64;
    const int64_t b = blockIdx.y;
    const int i = lane & 31, h = lane >> 5;
    // lane (i, h) feeds row row0 + 32 t + i of A and pool column i of V, k = 32 c + 16 h + 0..15 of chunk c
    const float* __restrict__ arow = A + (size_t)b * B * B + (size_t)(row0 + i) * B + 16 * h;
    const float* __restrict__ Vb = V + (size_t)b * B * POOL;
    const float* __restrict__ vcol = Vb + (size_t)i * B + 16 * h;
    v16f acc[2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
    struct Chunk { v4f a[2][4]; v4f v[4]; };
    auto load = [&](int c, Chunk& x) {
        const int k0 = 32 * c;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int u = 0; u < 4; ++u) x.a[t][u] = *reinterpret_cast<const v4f*>(arow + (size_t)(32 * t) * B + k0 + 4 * u);
#pragma unroll
        for (int u = 0; u < 4; ++u) x.v[u] = *reinterpret_cast<const v4f*>(vcol + k0 + 4 * u);
    };
    // MFMA step s contracts k = 32 c + 16 h + s on both operands
    auto mul = [&](const Chunk& x) {
#pragma unroll
        for (int s = 0; s < 16; ++s)
#pragma unroll
            for (int t = 0; t < 2; ++t)
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(x.a[t][s >> 2][s & 3], x.v[s >> 2][s & 3], acc[t], 0, 0, 0);
    };
    const int nchunks = B / 32;
    Chunk c0, c1;
    int c = wave;
    if (c < nchunks) load(c, c0);
    while (c < nchunks) {
        if (c + 4 < nchunks) load(c + 4, c1);
        mul(c0);
        c += 4;
        if (c >= nchunks) break;
        if (c + 4 < nchunks) load(c + 4, c0);
        mul(c1);
        c += 4;
    }
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) part[wave][t][r][lane] = acc[t][r];
    __syncthreads();
    // wavefront w finishes (tile, register group) pairs 2w and 2w+1: four consecutive rows of pool column i
    float* __restrict__ Wb = W + (size_t)b * B * POOL;
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int pq = 2 * wave + e, t = pq >> 2, q4 = pq & 3;
        const int row = row0 + 32 * t + 8 * q4 + 4 * h;
        const size_t off = (size_t)i * B + row;
        v4f out = *reinterpret_cast<const v4f*>(Vb + off);
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            float sum = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w) sum += part[w][t][4 * q4 + m][lane];
            out[m] = sum + eps * out[m];
        }
        *reinterpret_cast<v4f*>(Wb + off) = out;
    }
}

// grid = nblocks.  last != 0: also writes s = 2 max q, 1/s, s^(-1/p).  Eight threads per pool column.
__global__ __launch_bounds__(PNT) void pi_reduce_kernel(float* __restrict__ V, const float* __restrict__ W, int B,
                                                       float* __restrict__ q_out, int last, int p,
                                                       float* __restrict__ s, float* __restrict__ inv_s,
                                                       float* __restrict__ unscale) {
    __shared__ float qj[POOL];
    const int64_t b = blockIdx.x;
    const int j = threadIdx.x / 8, part = threadIdx.x % 8;
    float* __restrict__ Vc = V + (size_t)b * B * POOL + (size_t)j * B;
    const float* __restrict__ Wc = W + (size_t)b * B * POOL + (size_t)j * B;
    float nn = 0.f, vw = 0.f;
    for (int i = 4 * part; i < B; i += 32) {
        const v4f w = *reinterpret_cast<const v4f*>(Wc + i);
        const v4f v = *reinterpret_cast<const v4f*>(Vc + i);
#pragma unroll
        for (int m = 0; m < 4; ++m) { nn += w[m] * w[m]; vw += v[m] * w[m]; }
    }
    nn = sum8(nn);
    vw = sum8(vw);
    const float inv_norm = nn > 0.f ? 1.f / sqrtf(nn) : 0.f;
    if (part == 0) {
        qj[j] = vw;
        q_out[b * POOL + j] = vw;
    }
    for (int i = 4 * part; i < B; i += 32) {
        v4f w = *reinterpret_cast<const v4f*>(Wc + i);
#pragma unroll
        for (int m = 0; m < 4; ++m) w[m] *= inv_norm;
        *reinterpret_cast<v4f*>(Vc + i) = w;
    }
    __syncthreads();
    if (last && threadIdx.x == 0) {
        float best = qj[0];
        for (int c = 1; c < POOL; ++c) best = fmaxf(best, qj[c]);
        const float sv = 2.f * best;
        if (s) s[b] = sv;
        if (inv_s) inv_s[b] = 1.f / sv;
        if (unscale) unscale[b] = p == 2 ? 1.f / sqrtf(sv) : 1.f / sqrtf(sqrtf(sv));
    }
}

}  // namespace

size_t power_iteration_bytes_per_block(int B) { return 2 * (size_t)B * POOL * sizeof(float) + POOL * sizeof(float); }

hipError_t launch_power_iteration(const float* A, int64_t nblocks, int B, float eps, const float* V0, int pool,
                                  int sweeps, int p, float* V, float* W, float* q, float* s, float* inv_s,
                                  float* unscale, hipStream_t stream) {
    if (nblocks <= 0) return hipSuccess;
    if (pool < 1 || pool > POOL || sweeps < 1) return hipErrorInvalidValue;
    for (int64_t b0 = 0; b0 < nblocks; b0 += 65535) {
        const unsigned nb = (unsigned)(nblocks - b0 < 65535 ? nblocks - b0 : 65535);
        const size_t ov = (size_t)b0 * B * POOL;
        hipLaunchKernelGGL(pi_init_kernel, dim3(nb), dim3(PNT), 0, stream, V0, pool, B, V + ov);
        for (int t = 1; t <= sweeps; ++t) {
            hipLaunchKernelGGL(pi_sweep_kernel, dim3(B / 64, nb), dim3(PNT), 0, stream,
                               A + (size_t)b0 * B * B, V + ov, W + ov, B, eps);
            hipLaunchKernelGGL(pi_reduce_kernel, dim3(nb), dim3(PNT), 0, stream, V + ov, W + ov, B, q + b0 * POOL,
                               t == sweeps ? 1 : 0, p, s ? s + b0 : nullptr, inv_s ? inv_s + b0 : nullptr,
                               unscale ? unscale + b0 : nullptr);
        }
    }
    return hipGetLastError();
}

}  // namespace dash
