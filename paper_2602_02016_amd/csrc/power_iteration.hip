// Multi-Power-Iteration estimate of lambda_max for every block of a stack
// (paper Sections 3.4 and 3.5): a pool of up to 32 start vectors is multiplied by the
// block `sweeps` times, the largest Rayleigh quotient of the last sweep is lambda_PI, and
// the block is scaled by s = 2 * lambda_PI.
//
// One sweep reads the block once (4 B^2 bytes) and is HBM-bound, as the paper notes: the
// pool only widens the skinny product W = A V.  The pool vectors are kept pool-major
// ([32][B] per block: a column of V is contiguous) so that every operand of the sweep is
// read 16 bytes per lane.  Kernels:
//   pi_init    V_0 = start vectors with unit columns (pool padded with zero columns to 32); pi_spread copies it to every block
//   pi_sweep   W_b = A_b V_b + eps V_b with v_mfma_f32_32x32x2_f32, computed as W^T = V^T A (the
//              blocks are symmetric).  A workgroup owns 128 columns of A; its four wavefronts split
//              K (16-wide half-chunks, round robin), each streams its rows of the 128 columns
//              straight from global memory into the MFMA column operand -- 512 contiguous bytes
//              per half-wavefront and load, every element of A used once, no LDS staging -- and
//              reuses its chunk of V for the four column groups; the four partial results meet
//              in LDS.  The loads of a wavefront's next half-chunk are in flight while the MFMAs
//              of the current one run.
//              A sweep also leaves, per workgroup, the partial sums of |w_j|^2 and v_j . w_j of its
//              columns; the next sweep scales its input columns to unit length from them on the
//              way in, so no pass over the vectors lies between two sweeps.
//   pi_sweep16 the same sweep for pools of at most 16 vectors with v_mfma_f32_16x16x4_f32 (half the MFMA time)
//   pi_finalize  per block, after the last sweep: q_j = v_j . w_j, s = 2 max_j q_j, 1/s and s^(-1/p)
// Reductions are per block in a fixed order (no atomics): results do not depend on scheduling.
#include "kernels.h"

namespace dash {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));

namespace {

constexpr int POOL = 32;     // columns of V (pool members beyond the requested count are zero)
constexpr int PNT = 256;

// The start vectors are the same for every block: one workgroup per pool column writes the column, scaled to unit
// length, into block 0 of V (pool-major, [32][B]; columns beyond the requested m are zero), then every other block
// copies block 0.  grid = 32; V0: [B][m] row-major
__global__ __launch_bounds__(PNT) void pi_init_kernel(const float* __restrict__ V0, int m, int B,
                                                     float* __restrict__ V) {
    __shared__ float sh[PNT / 64];
    __shared__ float inv;
    const int c = blockIdx.x;
    float acc = 0.f;
    if (c < m)
        for (int i = threadIdx.x; i < B; i += PNT) { const float x = V0[(size_t)i * m + c]; acc += x * x; }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        float t = 0.f;
        for (int w = 0; w < PNT / 64; ++w) t += sh[w];
        inv = t > 0.f ? 1.f / sqrtf(t) : 0.f;
    }
    __syncthreads();
    const float sc = inv;
    for (int i = threadIdx.x; i < B; i += PNT) V[(size_t)c * B + i] = c < m ? V0[(size_t)i * m + c] * sc : 0.f;
}

// grid = (32 B / 4 / PNT, nblocks - 1): V_b = V_0 for b = 1 .. nblocks - 1
__global__ __launch_bounds__(PNT) void pi_spread_kernel(float* __restrict__ V, int B) {
    const size_t per = (size_t)B * POOL;
    const size_t f = (size_t)blockIdx.x * PNT + threadIdx.x;
    if (4 * f >= per) return;
    const v4f x = *reinterpret_cast<const v4f*>(V + 4 * f);
    *reinterpret_cast<v4f*>(V + ((size_t)blockIdx.y + 1) * per + 4 * f) = x;
}

// per-block scalars: q[32], then per workgroup of the sweep (128 columns each) the partial sums
// sum_n w[j][n]^2 and sum_n v[j][n] w[j][n] of its columns: [groups][2][32]
__host__ __device__ inline int pi_groups(int B) { return (B + 127) / 128; }
__host__ __device__ inline int pi_q_floats(int B) { return POOL + 2 * POOL * pi_groups(B); }

// grid = (B/128, nblocks); the four wavefronts of a workgroup split K.
// The blocks are symmetric, so W^T = V^T A: the pool is the MFMA's row operand and A its column operand,
// whose lane <-> column mapping lets a half-wavefront read 512 contiguous bytes of one row of A per load:
// lane (n', h) loads A[k][c0 + 4n' .. 4n'+3] for k = 16c + 8h + s (s = 0..7 within half-chunk c of 16 k) and
// feeds element m of the quad to the MFMA of column group m (columns c0 + 4n' + m, n' = 0..31); lane (j, h)
// supplies V[k][j] for the same k.  (For an input that is not exactly symmetric this is the power
// iteration of A^T, which has the same spectrum.)
// V holds the un-normalised product of the previous sweep; its columns are scaled to unit length on the
// way in, with the norms the previous sweep left as per-workgroup partial sums in qprev -- so a sweep is
// one launch, and it leaves its own partial sums (norms and Rayleigh quotients of its output) in qnext.
// STREAM: the stack is larger than the 256 MB last-level cache, so A is read with the non-temporal hint (+5 %)
template <bool STREAM>
__global__ __launch_bounds__(PNT, 2) void pi_sweep_kernel(const float* __restrict__ A, const float* __restrict__ V,
                                                         float* __restrict__ W, int B, float eps,
                                                         const float* __restrict__ qprev, float* __restrict__ qnext) {
    __shared__ float part[4][4][16][64];          // [wavefront][column group][accumulator register][lane]
    __shared__ float inv_norm[POOL];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c0 = blockIdx.x * 128;
    const int64_t b = blockIdx.y;
    const int i = lane & 31, h = lane >> 5;
    const int QF = pi_q_floats(B), NG = pi_groups(B);
    if (threadIdx.x < POOL) {
        const float* __restrict__ pp = qprev + b * QF + POOL;
        float nn = 0.f;
        for (int gidx = 0; gidx < NG; ++gidx) nn += pp[(size_t)gidx * 2 * POOL + threadIdx.x];
        inv_norm[threadIdx.x] = nn > 0.f ? 1.f / sqrtf(nn) : 0.f;
    }
    __syncthreads();
    const float my_inv = inv_norm[i];             // lane (j = i, h) feeds pool column i
    const bool valid = c0 + 4 * i < B;            // B is a multiple of 64: the last workgroup may own only 64 columns
    const float* __restrict__ acol = A + (size_t)b * B * B + (size_t)(8 * h) * B + c0 + 4 * i;
    const float* __restrict__ Vb = V + (size_t)b * B * POOL;
    const float* __restrict__ vrow = Vb + (size_t)i * B + 8 * h;
    v16f acc[4];
#pragma unroll
    for (int m = 0; m < 4; ++m)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[m][r] = 0.f;
    struct Half { v4f a[8]; v4f v[2]; };         // eight rows of A (a quad of columns each), eight k of V
    auto load = [&](int c, Half& x) {
        const int k0 = 16 * c;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            if (!valid) x.a[s] = v4f{0.f, 0.f, 0.f, 0.f};
            else if (STREAM) x.a[s] = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(acol + (size_t)(k0 + s) * B));
            else x.a[s] = *reinterpret_cast<const v4f*>(acol + (size_t)(k0 + s) * B);
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) x.v[u] = *reinterpret_cast<const v4f*>(vrow + k0 + 4 * u);
    };
    // MFMA step s contracts k = 16 c + 8 h + s on both operands
    auto mul = [&](const Half& x) {
#pragma unroll
        for (int s = 0; s < 8; ++s)
#pragma unroll
            for (int m = 0; m < 4; ++m)
                acc[m] = __builtin_amdgcn_mfma_f32_32x32x2f32(x.v[s >> 2][s & 3] * my_inv, x.a[s][m], acc[m], 0, 0, 0);
    };
    // half-chunks of 16 k, dealt round robin to the four wavefronts; the loads of a wavefront's next
    // half-chunk are in flight while the MFMAs of the current one run
    const int nhalf = B / 16;
    Half x0, x1;
    int c = wave;
    if (c < nhalf) load(c, x0);
    while (c < nhalf) {
        if (c + 4 < nhalf) load(c + 4, x1);
        mul(x0);
        c += 4;
        if (c >= nhalf) break;
        if (c + 4 < nhalf) load(c + 4, x0);
        mul(x1);
        c += 4;
    }
#pragma unroll
    for (int m = 0; m < 4; ++m)
#pragma unroll
        for (int r = 0; r < 16; ++r) part[wave][m][r][lane] = acc[m][r];
    __syncthreads();
    // accumulator register r of lane (n', h) is pool row j = 8 (r/4) + 4 h + r%4, column c0 + 4 n' + m of
    // group m: the four groups give a quad of consecutive columns.  Wavefront w finishes r = 4w .. 4w+3,
    // i.e. every pool row is finished by exactly one half-wavefront, which also sums its partials.
    float* __restrict__ Wb = W + (size_t)b * B * POOL;
    float* __restrict__ qn = qnext + b * QF + POOL + (size_t)blockIdx.x * 2 * POOL;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int r = 4 * wave + e;
        const int j = 8 * (r >> 2) + 4 * h + (r & 3);
        const size_t off = (size_t)j * B + c0 + 4 * i;
        float nn = 0.f, vw = 0.f;
        if (valid) {
            v4f vhat = *reinterpret_cast<const v4f*>(Vb + off);
            const float sj = inv_norm[j];
            v4f out;
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                float sum = 0.f;
#pragma unroll
                for (int w = 0; w < 4; ++w) sum += part[w][m][r][lane];
                vhat[m] *= sj;
                out[m] = sum + eps * vhat[m];
                nn += out[m] * out[m];
                vw += vhat[m] * out[m];
            }
            *reinterpret_cast<v4f*>(Wb + off) = out;
        }
#pragma unroll
        for (int d = 1; d < 32; d <<= 1) {
            nn += __shfl_xor(nn, d);
            vw += __shfl_xor(vw, d);
        }
        if (i == 0) {
            qn[j] = nn;
            qn[POOL + j] = vw;
        }
    }
}

// The same sweep for pools of at most 16 vectors, with v_mfma_f32_16x16x4_f32: half the matrix-core time per byte
// of A, which is what limits the 32-wide form (its 32 x 32 products need about as long as the block needs on
// HBM).  grid = (B/128, nblocks); the four wavefronts split K as above.  Lane (n', kq) of a wavefront loads, for
// the half-chunk c of 16 k, the quads A[16c + 4kq + s][c0 + 64 hf + 4n' .. + 3] (s = 0..3, hf = 0, 1: 256 contiguous
// bytes of four rows per load) and feeds element m of a quad to the MFMA of column group (hf, m); lane (j, kq)
// supplies V[16c + 4kq + s][j], a quad of consecutive k of the pool-major vector.  MFMA step s contracts
// k = 16c + 4kq + s over kq.  Accumulator register r of lane (n', kq) is pool row j = 4 kq + r, column
// c0 + 64 hf + 4n' + m: the four groups of a half give a quad of consecutive columns again.  Pool rows 16..31 of V
// and W are neither read nor written; their partial sums are written as zeros.
template <bool STREAM>
__global__ __launch_bounds__(PNT, 2) void pi_sweep16_kernel(const float* __restrict__ A, const float* __restrict__ V,
                                                           float* __restrict__ W, int B, float eps,
                                                           const float* __restrict__ qprev, float* __restrict__ qnext) {
    constexpr int P16 = 16;
    __shared__ float part[4][2][4][4][64];        // [wavefront][half][column group][accumulator register][lane]
    __shared__ float inv_norm[P16];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c0 = blockIdx.x * 128;
    const int64_t b = blockIdx.y;
    const int n = lane & 15, kq = lane >> 4;
    const int QF = pi_q_floats(B), NG = pi_groups(B);
    if (threadIdx.x < P16) {
        const float* __restrict__ pp = qprev + b * QF + POOL;
        float nn = 0.f;
        for (int gidx = 0; gidx < NG; ++gidx) nn += pp[(size_t)gidx * 2 * POOL + threadIdx.x];
        inv_norm[threadIdx.x] = nn > 0.f ? 1.f / sqrtf(nn) : 0.f;
    }
    __syncthreads();
    const float my_inv = inv_norm[n];             // lane (j = n, kq) feeds pool column n
    const bool valid1 = c0 + 64 < B;              // B is a multiple of 64: the last workgroup may own only 64 columns
    const float* __restrict__ acol = A + (size_t)b * B * B + (size_t)(4 * kq) * B + c0 + 4 * n;
    const float* __restrict__ Vb = V + (size_t)b * B * POOL;
    const float* __restrict__ vrow = Vb + (size_t)n * B + 4 * kq;
    v4f acc[2][4];
#pragma unroll
    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
        for (int m = 0; m < 4; ++m) acc[hf][m] = v4f{0.f, 0.f, 0.f, 0.f};
    struct Half { v4f a[2][4]; v4f v; };          // four rows of A (a quad of columns in each half), four k of V
    auto load = [&](int c, Half& x) {
        const int k0 = 16 * c;
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
                const float* p = acol + (size_t)(k0 + s) * B + 64 * hf;
                if (hf == 1 && !valid1) x.a[hf][s] = v4f{0.f, 0.f, 0.f, 0.f};
                else if (STREAM) x.a[hf][s] = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p));
                else x.a[hf][s] = *reinterpret_cast<const v4f*>(p);
            }
        x.v = *reinterpret_cast<const v4f*>(vrow + k0);
    };
    auto mul = [&](const Half& x) {
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int hf = 0; hf < 2; ++hf)
#pragma unroll
                for (int m = 0; m < 4; ++m)
                    acc[hf][m] = __builtin_amdgcn_mfma_f32_16x16x4f32(x.v[s] * my_inv, x.a[hf][s][m], acc[hf][m], 0, 0, 0);
    };
    const int nhalf = B / 16;
    Half x0, x1;
    int c = wave;
    if (c < nhalf) load(c, x0);
    while (c < nhalf) {
        if (c + 4 < nhalf) load(c + 4, x1);
        mul(x0);
        c += 4;
        if (c >= nhalf) break;
        if (c + 4 < nhalf) load(c + 4, x0);
        mul(x1);
        c += 4;
    }
#pragma unroll
    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
        for (int m = 0; m < 4; ++m)
#pragma unroll
            for (int r = 0; r < 4; ++r) part[wave][hf][m][r][lane] = acc[hf][m][r];
    __syncthreads();
    // wavefront w finishes accumulator register r = w: pool row j = 4 kq + w, one row per quarter-wavefront
    float* __restrict__ Wb = W + (size_t)b * B * POOL;
    float* __restrict__ qn = qnext + b * QF + POOL + (size_t)blockIdx.x * 2 * POOL;
    const int r = wave, j = 4 * kq + r;
    const float sj = inv_norm[j];
    float nn = 0.f, vw = 0.f;
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) {
        if (hf == 1 && !valid1) continue;
        const size_t off = (size_t)j * B + c0 + 64 * hf + 4 * n;
        v4f vhat = *reinterpret_cast<const v4f*>(Vb + off);
        v4f out;
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            float sum = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w) sum += part[w][hf][m][r][lane];
            vhat[m] *= sj;
            out[m] = sum + eps * vhat[m];
            nn += out[m] * out[m];
            vw += vhat[m] * out[m];
        }
        *reinterpret_cast<v4f*>(Wb + off) = out;
    }
#pragma unroll
    for (int d = 1; d < 16; d <<= 1) {
        nn += __shfl_xor(nn, d);
        vw += __shfl_xor(vw, d);
    }
    if (n == 0) {
        qn[j] = nn;
        qn[POOL + j] = vw;
    }
    if (threadIdx.x < POOL - P16) {               // the unused half of the pool
        qn[P16 + threadIdx.x] = 0.f;
        qn[POOL + P16 + threadIdx.x] = 0.f;
    }
}

// grid = nblocks: q_j = v_j . w_j of the last sweep (unit v), s = 2 max_j q_j, 1/s and s^(-1/p)
__global__ __launch_bounds__(64) void pi_finalize_kernel(float* __restrict__ qbuf, int B, int p, float* __restrict__ s,
                                                        float* __restrict__ inv_s, float* __restrict__ unscale) {
    const int64_t b = blockIdx.x;
    const int QF = pi_q_floats(B), NG = pi_groups(B);
    float* __restrict__ q = qbuf + b * QF;
    const int j = threadIdx.x;
    float vw = -3.0e38f;
    if (j < POOL) {
        vw = 0.f;
        for (int gidx = 0; gidx < NG; ++gidx) vw += q[POOL + (size_t)gidx * 2 * POOL + POOL + j];
        q[j] = vw;
    }
    float best = vw;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) best = fmaxf(best, __shfl_xor(best, d));
    if (j == 0) {
        const float sv = 2.f * best;
        if (s) s[b] = sv;
        if (inv_s) inv_s[b] = 1.f / sv;
        if (unscale) unscale[b] = p == 2 ? 1.f / sqrtf(sv) : 1.f / sqrtf(sqrtf(sv));
    }
}

// grid = nblocks: the start vectors are unit columns: norm partial 1 in group 0, 0 elsewhere
__global__ void pi_unit_norms_kernel(float* __restrict__ qbuf, int B) {
    const int QF = pi_q_floats(B), NG = pi_groups(B);
    float* __restrict__ q = qbuf + (size_t)blockIdx.x * QF + POOL;
    for (int t = threadIdx.x; t < 2 * POOL * NG; t += blockDim.x) q[t] = t < POOL ? 1.f : 0.f;
}

}  // namespace

size_t power_iteration_q_floats(int B) { return 2 * (size_t)pi_q_floats(B); }       // two buffers, ping-pong

size_t power_iteration_bytes_per_block(int B) {
    return 2 * (size_t)B * POOL * sizeof(float) + power_iteration_q_floats(B) * sizeof(float);
}

hipError_t launch_power_iteration(const float* A, int64_t nblocks, int B, float eps, const float* V0, int pool,
                                  int sweeps, int p, float* V, float* W, float* q, float* s, float* inv_s,
                                  float* unscale, hipStream_t stream) {
    if (nblocks <= 0) return hipSuccess;
    if (pool < 1 || pool > POOL || sweeps < 1) return hipErrorInvalidValue;
    const size_t QF = pi_q_floats(B);
    float* q0 = q;                                   // [nblocks][QF]
    float* q1 = q + (size_t)nblocks * QF;            // [nblocks][QF]
    for (int64_t b0 = 0; b0 < nblocks; b0 += 65535) {
        const unsigned nb = (unsigned)(nblocks - b0 < 65535 ? nblocks - b0 : 65535);
        const size_t ov = (size_t)b0 * B * POOL;
        float* src = V + ov;
        float* dst = W + ov;
        float* qa = q0 + b0 * QF;
        float* qb = q1 + b0 * QF;
        hipLaunchKernelGGL(pi_init_kernel, dim3(POOL), dim3(PNT), 0, stream, V0, pool, B, src);
        if (nb > 1)
            hipLaunchKernelGGL(pi_spread_kernel, dim3((unsigned)(((size_t)B * POOL / 4 + PNT - 1) / PNT), nb - 1), dim3(PNT), 0,
                               stream, src, B);
        hipLaunchKernelGGL(pi_unit_norms_kernel, dim3(nb), dim3(256), 0, stream, qa, B);
        for (int t = 1; t <= sweeps; ++t) {
            const bool big = (size_t)nblocks * B * B * sizeof(float) >= ((size_t)256 << 20);
            const dim3 grid((B + 127) / 128, nb);
            const float* Ab = A + (size_t)b0 * B * B;
            if (pool <= 16) {
                if (big) hipLaunchKernelGGL(pi_sweep16_kernel<true>, grid, dim3(PNT), 0, stream, Ab, src, dst, B, eps, qa, qb);
                else hipLaunchKernelGGL(pi_sweep16_kernel<false>, grid, dim3(PNT), 0, stream, Ab, src, dst, B, eps, qa, qb);
            } else {
                if (big) hipLaunchKernelGGL(pi_sweep_kernel<true>, grid, dim3(PNT), 0, stream, Ab, src, dst, B, eps, qa, qb);
                else hipLaunchKernelGGL(pi_sweep_kernel<false>, grid, dim3(PNT), 0, stream, Ab, src, dst, B, eps, qa, qb);
            }
            float* tv = src; src = dst; dst = tv;
            float* tq = qa; qa = qb; qb = tq;
        }
        // qa now holds the partial sums of the last sweep
        hipLaunchKernelGGL(pi_finalize_kernel, dim3(nb), dim3(64), 0, stream, qa, B, p, s ? s + b0 : nullptr,
                           inv_s ? inv_s + b0 : nullptr, unscale ? unscale + b0 : nullptr);
    }
    return hipGetLastError();
}

}  // namespace dash
