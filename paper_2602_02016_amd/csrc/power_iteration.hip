// Multi-Power-Iteration estimate of lambda_max for every block of a stack
// (paper Sections 3.4 and 3.5): a pool of up to 32 start vectors is multiplied by the
// block `sweeps` times, the largest Rayleigh quotient of the last sweep is lambda_PI, and
// the block is scaled by s = 2 * lambda_PI.
//
// One sweep reads the block once (4 B^2 bytes) and is HBM-bound, as the paper notes: the
// pool only widens the skinny product W = A V.  Kernels:
//   pi_init    V_b = start vectors with unit columns (pool padded with zero columns to 32)
//   pi_sweep   W_b = A_b V_b + eps V_b with v_mfma_f32_32x32x2_f32: a wavefront owns 32
//              rows of A; each lane streams 64 contiguous bytes of its row per 32-wide k
//              chunk straight from global memory into the MFMA A operand (every element
//              of A is used once, so LDS staging would buy nothing); the V operand (B x 32,
//              128 KB at B = 1024, shared by all wavefronts of the block) comes from L2
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

// grid = nblocks; V0: [B][m] row-major (shared by all blocks)
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
    for (int i = rg; i < B; i += PNT / POOL) Vb[(size_t)i * POOL + j] = j < m ? V0[(size_t)i * m + j] * inv_norm[j] : 0.f;
}

// grid = (ceil(B/128), nblocks); 4 wavefronts x 32 rows
__global__ __launch_bounds__(PNT) void pi_sweep_kernel(const float* __restrict__ A, const float* __restrict__ V,
                                                      float* __restrict__ W, int B, float eps) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row0 = blockIdx.x * 128 + wave * 32;
    if (row0 >= B) return;
    const int64_t b = blockIdx.y;
    const int i = lane & 31, h = lane >> 5;
    const float* __restrict__ arow = A + (size_t)b * B * B + (size_t)(row0 + i) * B + 16 * h;
    const float* __restrict__ Vb = V + (size_t)b * B * POOL;
    const float* __restrict__ vcol = Vb + (size_t)(16 * h) * POOL + i;     // i doubles as the pool index j
    v16f acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    // Two register sets: the loads of the next 32-wide k chunk are in flight while the 16 MFMAs of the
    // current one run (a wavefront is alone on its SIMD when the stack is short, so nothing else hides
    // the latency of its loads).  B is a multiple of 64: the number of chunks is even.
    v4f a0[4], a1[4];
    float v0[16], v1[16];
    auto load = [&](int k0, v4f (&a)[4], float (&v)[16]) {
#pragma unroll
        for (int u = 0; u < 4; ++u) a[u] = *reinterpret_cast<const v4f*>(arow + k0 + 4 * u);
#pragma unroll
        for (int s = 0; s < 16; ++s) v[s] = vcol[(size_t)(k0 + s) * POOL];
    };
    // MFMA step s contracts k = k0 + 16*h + s on both operands
    auto mul = [&](const v4f (&a)[4], const float (&v)[16]) {
#pragma unroll
        for (int s = 0; s < 16; ++s)
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[s >> 2][s & 3], v[s], acc, 0, 0, 0);
    };
    load(0, a0, v0);
    for (int k0 = 0; k0 < B; k0 += 64) {
        load(k0 + 32, a1, v1);
        mul(a0, v0);
        if (k0 + 64 < B) load(k0 + 64, a0, v0);
        mul(a1, v1);
    }
    float* __restrict__ Wb = W + (size_t)b * B * POOL;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int row = row0 + 8 * (r >> 2) + 4 * h + (r & 3);
        const size_t off = (size_t)row * POOL + i;
        Wb[off] = acc[r] + eps * Vb[off];
    }
}

// grid = nblocks.  last != 0: also writes s = 2 max q, 1/s, s^(-1/p).
__global__ __launch_bounds__(PNT) void pi_reduce_kernel(float* __restrict__ V, const float* __restrict__ W, int B,
                                                       float* __restrict__ q_out, int last, int p,
                                                       float* __restrict__ s, float* __restrict__ inv_s,
                                                       float* __restrict__ unscale) {
    __shared__ float pn[PNT / POOL][POOL], pq[PNT / POOL][POOL];
    __shared__ float inv_norm[POOL], qj[POOL];
    const int64_t b = blockIdx.x;
    const int j = threadIdx.x % POOL, rg = threadIdx.x / POOL;
    float* __restrict__ Vb = V + (size_t)b * B * POOL;
    const float* __restrict__ Wb = W + (size_t)b * B * POOL;
    float nn = 0.f, vw = 0.f;
    for (int i = rg; i < B; i += PNT / POOL) {
        const float w = Wb[(size_t)i * POOL + j];
        nn += w * w;
        vw += Vb[(size_t)i * POOL + j] * w;
    }
    pn[rg][j] = nn;
    pq[rg][j] = vw;
    __syncthreads();
    if (rg == 0) {
        float tn = 0.f, tq = 0.f;
        for (int r = 0; r < PNT / POOL; ++r) { tn += pn[r][j]; tq += pq[r][j]; }
        inv_norm[j] = tn > 0.f ? 1.f / sqrtf(tn) : 0.f;
        qj[j] = tq;
        q_out[b * POOL + j] = tq;
    }
    __syncthreads();
    for (int i = rg; i < B; i += PNT / POOL) Vb[(size_t)i * POOL + j] = Wb[(size_t)i * POOL + j] * inv_norm[j];
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
            hipLaunchKernelGGL(pi_sweep_kernel, dim3((B + 127) / 128, nb), dim3(PNT), 0, stream,
                               A + (size_t)b0 * B * B, V + ov, W + ov, B, eps);
            hipLaunchKernelGGL(pi_reduce_kernel, dim3(nb), dim3(PNT), 0, stream, V + ov, W + ov, B, q + b0 * POOL,
                               t == sweeps ? 1 : 0, p, s ? s + b0 : nullptr, inv_s ? inv_s + b0 : nullptr,
                               unscale ? unscale + b0 : nullptr);
        }
    }
    return hipGetLastError();
}

}  // namespace dash
