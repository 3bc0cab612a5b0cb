// HBM-bound kernels of the path: per-block Frobenius norm / trace (paper Section 3.4),
// the closed-form first Newton-DB iterate and the Chebyshev start terms (Section 3.3,
// Appendix A.2), and block-wise Adam grafting (Section 2.3).
//
// All of them stream the stack once with 16-byte accesses, 256 threads per workgroup,
// one workgroup per row slab of a block so that even a short stack gives the 256 CUs
// enough workgroups.  Per-block reductions are two-stage (slab partials, then a fixed
// order sum) so results do not depend on scheduling; no atomics are used.
#include "kernels.h"

namespace dash {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef unsigned short v4s __attribute__((ext_vector_type(4)));

// fp32 -> 16-bit operand format, round to nearest even
__device__ __forceinline__ unsigned short to_half(float v, int half) {
    if (half == HALF_FP16) { union { _Float16 h; unsigned short u; } x; x.h = (_Float16)v; return x.u; }
    union { __bf16 h; unsigned short u; } x; x.h = (__bf16)v; return x.u;
}

__device__ __forceinline__ float from_half(unsigned short u, int half) {
    if (half == HALF_FP16) { union { _Float16 h; unsigned short u; } x; x.u = u; return (float)x.h; }
    union { __bf16 h; unsigned short u; } x; x.u = u; return (float)x.h;
}

constexpr int NT = 256;

// Streaming accesses.  S = true: the call touches more bytes than the last-level cache holds (256 MB) and every
// byte once, so quads are read and written with the non-temporal hint; with it, and with each workgroup walking one contiguous range
// in passes of UNR x NT quads, a read-modify-write stream over 1 GiB arrays measured 5.8-6.0 TB/s against 4.5-4.8
// for a grid-stride loop with plain accesses (a read-only stream: 6.4-6.7).
constexpr int UNR = 4;
constexpr size_t STREAM_BYTES = (size_t)256 << 20;
template <bool S> __device__ __forceinline__ v4f ldq(const float* p) {
    return S ? __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p)) : *reinterpret_cast<const v4f*>(p);
}
template <bool S> __device__ __forceinline__ void stq(float* p, v4f v) {
    if (S) __builtin_nontemporal_store(v, reinterpret_cast<v4f*>(p)); else *reinterpret_cast<v4f*>(p) = v;
}

int norm_slabs(int B) { return B >= 256 ? 32 : 8; }   // B is a multiple of 64, so both divide B

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// sum over the workgroup; result valid in thread 0
__device__ __forceinline__ float block_sum(float v, float* sh) {
    v = wave_sum(v);
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    if (lane == 0) sh[w] = v;
    __syncthreads();
    float r = 0.f;
    if (threadIdx.x == 0) {
#pragma unroll
        for (int i = 0; i < NT / 64; ++i) r += sh[i];
    }
    __syncthreads();
    return r;
}

// grid = (P, nblocks): slab q of block b
template <bool S>
__global__ __launch_bounds__(NT) void norm_partials_kernel(const float* __restrict__ A, int B, int P,
                                                          float eps, int mode, float* __restrict__ partial) {
    __shared__ float sh[NT / 64];
    const int q = blockIdx.x;
    const int64_t b = blockIdx.y;
    const int rows = B / P, r0 = q * rows;
    const float* __restrict__ Ab = A + (size_t)b * B * B;
    float acc = 0.f;
    if (mode == 0) {
        const int qpr = B / 4;   // float4 per row
        const int cnt = rows * qpr;                       // the slab is contiguous: quad f at r0 * B + 4 f
        const float* __restrict__ slab = Ab + (size_t)r0 * B;
        for (int f0 = threadIdx.x; f0 < cnt; f0 += UNR * NT) {
            v4f v[UNR];
#pragma unroll
            for (int u = 0; u < UNR; ++u)
                if (f0 + u * NT < cnt) v[u] = ldq<S>(slab + 4 * (size_t)(f0 + u * NT));
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                const int f = f0 + u * NT;
                if (f < cnt) {
                    const int r = r0 + f / qpr, c = 4 * (f % qpr);
                    if (r >= c && r < c + 4) v[u][r - c] += eps;
                    acc += v[u][0] * v[u][0] + v[u][1] * v[u][1] + v[u][2] * v[u][2] + v[u][3] * v[u][3];
                }
            }
        }
    } else {
        for (int r = r0 + threadIdx.x; r < r0 + rows; r += NT) acc += Ab[(size_t)r * B + r] + eps;
    }
    const float tot = block_sum(acc, sh);
    if (threadIdx.x == 0) partial[b * P + q] = tot;
}

__global__ void finalize_scale_kernel(const float* __restrict__ partial, int64_t n, int P, int mode, int p,
                                      float* s, float* inv_s, float* unscale) {
    const int64_t b = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (b >= n) return;
    float sv = 1.f;
    if (mode != 2) {
        float t = 0.f;
        for (int q = 0; q < P; ++q) t += partial[b * P + q];
        sv = mode == 0 ? sqrtf(t) : t;
    }
    if (s) s[b] = sv;
    if (inv_s) inv_s[b] = 1.f / sv;
    if (unscale) unscale[b] = p == 2 ? 1.f / sqrtf(sv) : 1.f / sqrtf(sqrtf(sv));
}

// grid = (B*B/4/NT per block ..., nblocks) flattened over blockIdx.x within a block
__global__ __launch_bounds__(NT) void scale_shift_kernel(const float* __restrict__ in, int B, float eps,
                                                        const float* __restrict__ mult, float a1, float g1,
                                                        float* __restrict__ out1, float a2, float g2,
                                                        float* __restrict__ out2, unsigned short* __restrict__ h1,
                                                        unsigned short* __restrict__ h2, int32_t* nonfinite, int half,
                                                        unsigned short* __restrict__ l1,
                                                        unsigned short* __restrict__ l2,
                                                        unsigned short* __restrict__ ll1,
                                                        unsigned short* __restrict__ ll2) {
    const int64_t b = blockIdx.y;
    const int f = blockIdx.x * NT + threadIdx.x;     // float4 index inside the block
    const int qpr = B / 4;
    if (f >= B * qpr) return;
    const int r = f / qpr, c = 4 * (f % qpr);
    const size_t off = (size_t)b * B * B + (size_t)r * B + c;
    const float m = mult ? mult[b] : 1.f;
    v4f v = *reinterpret_cast<const v4f*>(in + off);
    const int d = r - c;                              // diagonal position inside this float4, if 0..3
    if (d >= 0 && d < 4) v[d] += eps;
    v4f o1, o2;
    bool bad = false;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        o1[i] = a1 * (v[i] * m) + (i == d ? g1 : 0.f);
        o2[i] = a2 * o1[i] + (i == d ? g2 : 0.f);
        bad |= !(fabsf(o1[i]) <= 3.0e38f);
    }
    if (out1) *reinterpret_cast<v4f*>(out1 + off) = o1;
    if (out2) *reinterpret_cast<v4f*>(out2 + off) = o2;
    if (h1) {
        v4s t;
#pragma unroll
        for (int i = 0; i < 4; ++i) t[i] = to_half(o1[i], half);
        *reinterpret_cast<v4s*>(h1 + off) = t;
    }
    if (h2) {
        v4s t;
#pragma unroll
        for (int i = 0; i < 4; ++i) t[i] = to_half(o2[i], half);
        *reinterpret_cast<v4s*>(h2 + off) = t;
    }
    // low planes of the split representation x ~ hi + lo, lo = round(x - hi); with two fp16 planes the low plane is
    // stored times 2^11 (it would go subnormal otherwise; the matmul kernel scales the sum of its segments back)
    const float ls1 = (half == HALF_FP16 && !ll1) ? 2048.f : 1.f, ls2 = (half == HALF_FP16 && !ll2) ? 2048.f : 1.f;
    if (l1) {
        v4s t;
#pragma unroll
        for (int i = 0; i < 4; ++i) t[i] = to_half((o1[i] - from_half(to_half(o1[i], half), half)) * ls1, half);
        *reinterpret_cast<v4s*>(l1 + off) = t;
    }
    if (l2) {
        v4s t;
#pragma unroll
        for (int i = 0; i < 4; ++i) t[i] = to_half((o2[i] - from_half(to_half(o2[i], half), half)) * ls2, half);
        *reinterpret_cast<v4s*>(l2 + off) = t;
    }
    // third planes, x ~ hi + mid + lo: lo = round(x - hi - mid)
    if (ll1) {
        v4s t;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float r1 = o1[i] - from_half(to_half(o1[i], half), half);
            t[i] = to_half(r1 - from_half(to_half(r1, half), half), half);
        }
        *reinterpret_cast<v4s*>(ll1 + off) = t;
    }
    if (ll2) {
        v4s t;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float r2 = o2[i] - from_half(to_half(o2[i], half), half);
            t[i] = to_half(r2 - from_half(to_half(r2, half), half), half);
        }
        *reinterpret_cast<v4s*>(ll2 + off) = t;
    }
    if (nonfinite && bad) nonfinite[b] = 1;
}

__global__ void fill_i32_kernel(int32_t* p, int64_t n, int32_t v) {
    const int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// grid = (P, nblocks)
template <bool S>
__global__ __launch_bounds__(NT) void graft_partials_kernel(const float* __restrict__ G, const float* __restrict__ U,
                                                           float* __restrict__ Acc, int64_t elems, int P, float beta_g,
                                                           float eps_g, float* __restrict__ partial) {
    __shared__ float sh[NT / 64];
    const int q = blockIdx.x;
    const int64_t b = blockIdx.y;
    const size_t per = (size_t)elems / P;             // contiguous floats per slab
    const size_t base = (size_t)b * elems + (size_t)q * per;
    float sp = 0.f, su = 0.f;
    const size_t cnt = per / 4;
    for (size_t f0 = threadIdx.x; f0 < cnt; f0 += UNR * NT) {
        v4f g[UNR], u[UNR], a[UNR];
#pragma unroll
        for (int k = 0; k < UNR; ++k)
            if (f0 + k * NT < cnt) {
                const size_t off = base + 4 * (f0 + k * NT);
                g[k] = ldq<S>(G + off);
                u[k] = ldq<S>(U + off);
                a[k] = ldq<S>(Acc + off);
            }
#pragma unroll
        for (int k = 0; k < UNR; ++k)
            if (f0 + k * NT < cnt) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    a[k][i] = beta_g * a[k][i] + (1.f - beta_g) * g[k][i] * g[k][i];
                    const float pv = g[k][i] / (eps_g + sqrtf(a[k][i]));
                    sp += pv * pv;
                    su += u[k][i] * u[k][i];
                }
                stq<S>(Acc + base + 4 * (f0 + k * NT), a[k]);
            }
    }
    const float tp = block_sum(sp, sh);
    const float tu = block_sum(su, sh);
    if (threadIdx.x == 0) {
        partial[(b * P + q) * 2 + 0] = tp;
        partial[(b * P + q) * 2 + 1] = tu;
    }
}

// grid = (P, nblocks)
// theta -= lr * s_b * U (theta may be null); scaled = s_b * U (scaled may be null, may equal U)
template <bool S>
__global__ __launch_bounds__(NT) void graft_apply_kernel(const float* U, float* __restrict__ theta,
                                                        const float* __restrict__ partial, int64_t elems, int P, float lr,
                                                        float* __restrict__ s_out, float* scaled) {
    const int q = blockIdx.x;
    const int64_t b = blockIdx.y;
    float tp = 0.f, tu = 0.f;
    for (int i = 0; i < P; ++i) {
        tp += partial[(b * P + i) * 2 + 0];
        tu += partial[(b * P + i) * 2 + 1];
    }
    // a block whose update is all zero (a gradient block that saw no data) has nothing to scale: s = 0, not 0/0
    const float s = tu > 0.f ? sqrtf(tp) / sqrtf(tu) : 0.f;
    if (s_out && q == 0 && threadIdx.x == 0) s_out[b] = s;
    if (!theta && !scaled) return;
    const float k = lr * s;
    const size_t per = (size_t)elems / P;
    const size_t base = (size_t)b * elems + (size_t)q * per;
    const size_t cnt = per / 4;
    for (size_t f0 = threadIdx.x; f0 < cnt; f0 += UNR * NT) {
        v4f u[UNR], t[UNR];
#pragma unroll
        for (int j = 0; j < UNR; ++j)
            if (f0 + j * NT < cnt) {
                const size_t off = base + 4 * (f0 + j * NT);
                u[j] = ldq<S>(U + off);
                if (theta) t[j] = ldq<S>(theta + off);
            }
#pragma unroll
        for (int j = 0; j < UNR; ++j)
            if (f0 + j * NT < cnt) {
                const size_t off = base + 4 * (f0 + j * NT);
                if (theta) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) t[j][i] -= k * u[j][i];
                    stq<S>(theta + off, t[j]);
                }
                if (scaled) {
                    v4f w;
#pragma unroll
                    for (int i = 0; i < 4; ++i) w[i] = s * u[j][i];
                    stq<S>(scaled + off, w);
                }
            }
    }
}

// y -= a * x over n floats (16-byte aligned): every workgroup takes contiguous ranges of UNR x NT quads, one per pass
template <bool S>
__global__ __launch_bounds__(NT) void axpy_kernel(float* __restrict__ y, const float* __restrict__ x, int64_t n, float a) {
    const int64_t n4 = n / 4;
    if (blockIdx.x == 0 && threadIdx.x < (unsigned)(n - 4 * n4)) {      // the up to three elements past the quads
        const int64_t e = 4 * n4 + threadIdx.x;
        y[e] -= a * x[e];
    }
    const int64_t per = (int64_t)UNR * NT;
    for (int64_t c = blockIdx.x; c * per < n4; c += gridDim.x) {
        const int64_t f0 = c * per + threadIdx.x;
        v4f u[UNR], t[UNR];
#pragma unroll
        for (int q = 0; q < UNR; ++q)
            if (f0 + q * NT < n4) {
                u[q] = ldq<S>(x + 4 * (f0 + q * NT));
                t[q] = ldq<S>(y + 4 * (f0 + q * NT));
            }
#pragma unroll
        for (int q = 0; q < UNR; ++q)
            if (f0 + q * NT < n4) {
#pragma unroll
                for (int i = 0; i < 4; ++i) t[q][i] -= a * u[q][i];
                stq<S>(y + 4 * (f0 + q * NT), t[q]);
            }
    }
}

// ---- 1-D parameters (normalisation layers, paper Section 4.1): the gradient block is a vector ----
// L_b <- beta L_b + alpha g_b g_b^T ; grid = (B*B/4/NT, nblocks)
__global__ __launch_bounds__(NT) void outer_accumulate_kernel(const float* __restrict__ g, float* __restrict__ L, int B,
                                                             float beta, float alpha) {
    const int64_t b = blockIdx.y;
    const int f = blockIdx.x * NT + threadIdx.x;
    const int qpr = B / 4;
    if (f >= B * qpr) return;
    const int r = f / qpr, c = 4 * (f % qpr);
    const float* __restrict__ gb = g + (size_t)b * B;
    const float gi = alpha * gb[r];
    const v4f gj = *reinterpret_cast<const v4f*>(gb + c);
    float* __restrict__ p = L + (size_t)b * B * B + (size_t)r * B + c;
    v4f l = *reinterpret_cast<const v4f*>(p);
#pragma unroll
    for (int i = 0; i < 4; ++i) l[i] = beta * l[i] + gi * gj[i];
    *reinterpret_cast<v4f*>(p) = l;
}

// u_b = X_b g_b ; grid = (B/16, nblocks); each of the 4 wavefronts of a workgroup owns 4 rows,
// lanes stride along the row with 16-byte loads, wavefront shuffle reduction
__global__ __launch_bounds__(NT) void matvec_kernel(const float* __restrict__ X, const float* __restrict__ g,
                                                   float* __restrict__ u, int B) {
    const int64_t b = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float* __restrict__ gb = g + (size_t)b * B;
    for (int rr = 0; rr < 4; ++rr) {
        const int r = blockIdx.x * 16 + wave * 4 + rr;
        const float* __restrict__ xr = X + (size_t)b * B * B + (size_t)r * B;
        float acc = 0.f;
        for (int k = 4 * lane; k < B; k += 256) {
            const v4f x = *reinterpret_cast<const v4f*>(xr + k);
            const v4f v = *reinterpret_cast<const v4f*>(gb + k);
            acc += x[0] * v[0] + x[1] * v[1] + x[2] * v[2] + x[3] * v[3];
        }
        acc = wave_sum(acc);
        if (lane == 0) u[(size_t)b * B + r] = acc;
    }
}

// ---- block() / its inverse (paper Section 4.1): sub-matrices of a row-major layer <-> a stack ----
// stack[(im*nn + in)][r][c] <-> W[(r0 + im*B + r) * ld + c0 + in*B + c], r < bm, c < bn.  A stack block is
// pm x pn >= bm x bn: gathering fills the padding with zeros, scattering ignores it.
// VEC = 4: 16-byte accesses (needs ld, c0, B, bn, pn multiples of 4 and aligned bases); VEC = 1: any shape.
// grid = (ceil(pm*pn/VEC / NT), nm*nn)
template <int VEC, bool SCATTER>
__global__ __launch_bounds__(NT) void block_copy_kernel(float* __restrict__ W, float* __restrict__ stack, int64_t ld,
                                                       int64_t r0, int64_t c0, int B, int bm, int bn, int pm, int pn,
                                                       int nn) {
    const int64_t blk = blockIdx.y;
    const int64_t im = blk / nn, in = blk % nn;
    const int per_row = pn / VEC;
    const int64_t f = (int64_t)blockIdx.x * NT + threadIdx.x;
    if (f >= (int64_t)pm * per_row) return;
    const int r = (int)(f / per_row), c = (int)(f % per_row) * VEC;
    const bool inside = r < bm && c < bn;              // bn is a multiple of VEC: a quad is inside or outside
    float* w = W + (r0 + im * B + r) * ld + c0 + in * B + c;
    float* s = stack + blk * pm * pn + (int64_t)r * pn + c;
    if (VEC == 4) {
        if (SCATTER) {
            if (inside) *reinterpret_cast<v4f*>(w) = *reinterpret_cast<const v4f*>(s);
        } else {
            v4f v = {0.f, 0.f, 0.f, 0.f};
            if (inside) v = *reinterpret_cast<const v4f*>(w);
            *reinterpret_cast<v4f*>(s) = v;
        }
    } else {
        if (SCATTER) {
            if (inside) *w = *s;
        } else {
            *s = inside ? *w : 0.f;
        }
    }
}

// ---- launchers ------------------------------------------------------------------------


hipError_t launch_norm_partials(const float* A, int64_t nblocks, int B, float eps, int mode, float* partial,
                                hipStream_t stream) {
    const int P = norm_slabs(B);
    for (int64_t b0 = 0; b0 < nblocks; b0 += 65535) {
        const int64_t nb = nblocks - b0 < 65535 ? nblocks - b0 : 65535;
        if ((size_t)nblocks * B * B * 4 >= STREAM_BYTES)
            hipLaunchKernelGGL(norm_partials_kernel<true>, dim3(P, (unsigned)nb), dim3(NT), 0, stream,
                               A + (size_t)b0 * B * B, B, P, eps, mode, partial + b0 * P);
        else
            hipLaunchKernelGGL(norm_partials_kernel<false>, dim3(P, (unsigned)nb), dim3(NT), 0, stream,
                               A + (size_t)b0 * B * B, B, P, eps, mode, partial + b0 * P);
    }
    return hipGetLastError();
}

hipError_t launch_finalize_scale(const float* partial, int64_t nblocks, int P, int mode, int p, float* s,
                                 float* inv_s, float* unscale, hipStream_t stream) {
    if (nblocks <= 0) return hipSuccess;
    hipLaunchKernelGGL(finalize_scale_kernel, dim3((unsigned)((nblocks + 255) / 256)), dim3(256), 0, stream,
                       partial, nblocks, P, mode, p, s, inv_s, unscale);
    return hipGetLastError();
}

hipError_t launch_scale_shift(const float* in, int64_t nblocks, int B, float eps, const float* mult, float a1,
                              float g1, float* out1, float a2, float g2, float* out2, void* h1, void* h2,
                              int32_t* nonfinite, hipStream_t stream, int half, void* l1, void* l2, void* ll1,
                              void* ll2) {
    const unsigned gx = (unsigned)(((size_t)B * B / 4 + NT - 1) / NT);
    for (int64_t b0 = 0; b0 < nblocks; b0 += 65535) {
        const int64_t nb = nblocks - b0 < 65535 ? nblocks - b0 : 65535;
        const size_t o = (size_t)b0 * B * B;
        hipLaunchKernelGGL(scale_shift_kernel, dim3(gx, (unsigned)nb), dim3(NT), 0, stream, in + o, B, eps,
                           mult ? mult + b0 : nullptr, a1, g1, out1 ? out1 + o : nullptr, a2, g2,
                           out2 ? out2 + o : nullptr, h1 ? static_cast<unsigned short*>(h1) + o : nullptr,
                           h2 ? static_cast<unsigned short*>(h2) + o : nullptr, nonfinite ? nonfinite + b0 : nullptr,
                           half, l1 ? static_cast<unsigned short*>(l1) + o : nullptr,
                           l2 ? static_cast<unsigned short*>(l2) + o : nullptr,
                           ll1 ? static_cast<unsigned short*>(ll1) + o : nullptr,
                           ll2 ? static_cast<unsigned short*>(ll2) + o : nullptr);
    }
    return hipGetLastError();
}

hipError_t launch_outer_accumulate(const float* g, float* L, int64_t nblocks, int B, float beta, float alpha,
                                   hipStream_t stream) {
    const unsigned gx = (unsigned)(((size_t)B * B / 4 + NT - 1) / NT);
    for (int64_t b0 = 0; b0 < nblocks; b0 += 65535) {
        const int64_t nb = nblocks - b0 < 65535 ? nblocks - b0 : 65535;
        hipLaunchKernelGGL(outer_accumulate_kernel, dim3(gx, (unsigned)nb), dim3(NT), 0, stream, g + (size_t)b0 * B,
                           L + (size_t)b0 * B * B, B, beta, alpha);
    }
    return hipGetLastError();
}

hipError_t launch_matvec(const float* X, const float* g, float* u, int64_t nblocks, int B, hipStream_t stream) {
    for (int64_t b0 = 0; b0 < nblocks; b0 += 65535) {
        const int64_t nb = nblocks - b0 < 65535 ? nblocks - b0 : 65535;
        hipLaunchKernelGGL(matvec_kernel, dim3(B / 16, (unsigned)nb), dim3(NT), 0, stream, X + (size_t)b0 * B * B,
                           g + (size_t)b0 * B, u + (size_t)b0 * B, B);
    }
    return hipGetLastError();
}

hipError_t launch_block_copy(float* W, float* stack, int64_t ld, int64_t r0, int64_t c0, int B, int bm, int bn,
                             int pm, int pn, int64_t nm, int64_t nn, bool scatter, hipStream_t stream) {
    if (nm <= 0 || nn <= 0 || bm <= 0 || bn <= 0) return hipSuccess;
    if (nn > 0x7fffffff || pm < bm || pn < bn) return hipErrorInvalidValue;
    const bool vec = ld % 4 == 0 && c0 % 4 == 0 && B % 4 == 0 && bn % 4 == 0 && pn % 4 == 0 &&
                     (uintptr_t)W % 16 == 0 && (uintptr_t)stack % 16 == 0;
    const int V = vec ? 4 : 1;
    const unsigned gx = (unsigned)(((int64_t)pm * (pn / V) + NT - 1) / NT);
    // grid.y is limited to 65535: whole rows of blocks per launch (all of them in the usual case)
    const int64_t rows_per = nn > 65535 ? 0 : 65535 / nn;
    if (rows_per == 0) return hipErrorInvalidValue;
    for (int64_t m0 = 0; m0 < nm; m0 += rows_per) {
        const int64_t mr = nm - m0 < rows_per ? nm - m0 : rows_per;
        dim3 grid(gx, (unsigned)(mr * nn)), block(NT);
        float* st = stack + m0 * nn * pm * pn;
        const int64_t rr = r0 + m0 * B;
        if (vec && scatter) hipLaunchKernelGGL((block_copy_kernel<4, true>), grid, block, 0, stream, W, st, ld, rr, c0, B, bm, bn, pm, pn, (int)nn);
        else if (vec) hipLaunchKernelGGL((block_copy_kernel<4, false>), grid, block, 0, stream, W, st, ld, rr, c0, B, bm, bn, pm, pn, (int)nn);
        else if (scatter) hipLaunchKernelGGL((block_copy_kernel<1, true>), grid, block, 0, stream, W, st, ld, rr, c0, B, bm, bn, pm, pn, (int)nn);
        else hipLaunchKernelGGL((block_copy_kernel<1, false>), grid, block, 0, stream, W, st, ld, rr, c0, B, bm, bn, pm, pn, (int)nn);
    }
    return hipGetLastError();
}

hipError_t launch_fill_i32(int32_t* p, int64_t n, int32_t v, hipStream_t stream) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, p, n, v);
    return hipGetLastError();
}

// slabs a block of `elems` floats is cut into for the grafting reductions (each a multiple of 4 floats)
int graft_slabs(int64_t elems) { return elems >= 65536 ? 32 : elems >= 4096 ? 8 : 1; }

hipError_t launch_graft_partials(const float* G, const float* U, float* Acc, int64_t nblocks, int64_t elems,
                                 float beta_g, float eps_g, float* partial, hipStream_t stream) {
    const int P = graft_slabs(elems);
    if (elems % (4 * P)) return hipErrorInvalidValue;
    for (int64_t b0 = 0; b0 < nblocks; b0 += 65535) {
        const int64_t nb = nblocks - b0 < 65535 ? nblocks - b0 : 65535;
        const size_t o = (size_t)b0 * elems;
        if ((size_t)nblocks * elems * 16 >= STREAM_BYTES)
            hipLaunchKernelGGL(graft_partials_kernel<true>, dim3(P, (unsigned)nb), dim3(NT), 0, stream, G + o, U + o,
                               Acc + o, elems, P, beta_g, eps_g, partial + b0 * P * 2);
        else
            hipLaunchKernelGGL(graft_partials_kernel<false>, dim3(P, (unsigned)nb), dim3(NT), 0, stream, G + o, U + o,
                               Acc + o, elems, P, beta_g, eps_g, partial + b0 * P * 2);
    }
    return hipGetLastError();
}

hipError_t launch_graft_apply(const float* U, float* theta, const float* partial, int64_t nblocks, int64_t elems,
                              float lr, float* s_out, float* scaled, hipStream_t stream) {
    const int P = graft_slabs(elems);
    if (elems % (4 * P)) return hipErrorInvalidValue;
    for (int64_t b0 = 0; b0 < nblocks; b0 += 65535) {
        const int64_t nb = nblocks - b0 < 65535 ? nblocks - b0 : 65535;
        const size_t o = (size_t)b0 * elems;
        if ((size_t)nblocks * elems * 12 >= STREAM_BYTES)
            hipLaunchKernelGGL(graft_apply_kernel<true>, dim3(P, (unsigned)nb), dim3(NT), 0, stream, U + o,
                               theta ? theta + o : nullptr, partial + b0 * P * 2, elems, P, lr,
                               s_out ? s_out + b0 : nullptr, scaled ? scaled + o : nullptr);
        else
            hipLaunchKernelGGL(graft_apply_kernel<false>, dim3(P, (unsigned)nb), dim3(NT), 0, stream, U + o,
                               theta ? theta + o : nullptr, partial + b0 * P * 2, elems, P, lr,
                               s_out ? s_out + b0 : nullptr, scaled ? scaled + o : nullptr);
    }
    return hipGetLastError();
}

hipError_t launch_axpy(float* y, const float* x, int64_t n, float a, hipStream_t stream) {
    if (n <= 0) return hipSuccess;
    const int64_t chunks = (n / 4 + UNR * NT - 1) / (UNR * NT);
    const dim3 grid((unsigned)(chunks < 1 ? 1 : chunks < 1024 ? chunks : 1024));
    if ((size_t)n * 12 >= STREAM_BYTES) hipLaunchKernelGGL(axpy_kernel<true>, grid, dim3(NT), 0, stream, y, x, n, a);
    else hipLaunchKernelGGL(axpy_kernel<false>, grid, dim3(NT), 0, stream, y, x, n, a);
    return hipGetLastError();
}

}  // namespace dash
